// Shared declarations of the gfx950 kernels: tile layout of the private int8
// buffers, fp16 bit helpers, launcher prototypes.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <atomic>

namespace llmint8 {

// ---- private int8 layout ---------------------------------------------------
// A matrix M[rows][K] of int8 (rows = tokens of X, or output columns of W;
// K = features) is cut into tiles of 32 rows x 32 features.  A tile is 1 KiB
// stored in the operand order of v_mfma_i32_32x32x32_i8: lane l of a wave
// holds row (l % 32), features 16*(l / 32) .. +15, so byte (r, kk) of a tile
// sits at ((kk >> 4) * 32 + r) * 16 + (kk & 15).  Tiles of one row block are
// consecutive along K: tile (rt, kt) starts at (rt * KT + kt) * 1024 with
// KT = 4 * ceil(h / 128).  Rows and features beyond the matrix are zero.
constexpr int TILE = 32;
constexpr int TILE_BYTES = 1024;

__host__ __device__ inline int k_tiles(int h) { return 4 * ((h + 127) / 128); }
__host__ __device__ inline int row_tiles(int n) { return (n + 31) / 32; }
__host__ __device__ inline int tile_byte(int r, int kk) { return (((kk >> 4) << 5) + r) * 16 + (kk & 15); }
__host__ __device__ inline int opad_of(int cap) { return (cap + 15) & ~15; }

// ---- fp16 as bit patterns ----------------------------------------------------
// For finite values the magnitude order of binary16 equals the integer order
// of (bits & 0x7fff), so absolute maxima and the threshold test are done on
// integers and are exact.
__device__ inline float f16_bits_to_float(unsigned short b)
{
    return (float)__builtin_bit_cast(_Float16, b);  // exact widening
}

// hi - lo of a zeropoint record's first word (fp16 bits of lo in the low half, of hi in the high half): exact
__device__ inline double zp_range(unsigned lohi)
{
    return (double)f16_bits_to_float((unsigned short)(lohi >> 16)) -
           (double)f16_bits_to_float((unsigned short)(lohi & 0xffffu));
}

// ---- zeropoint quantization (Section 2.1, Eq. 1-3), shared by the kernels of zeropoint.hip and the
// short-X pre-pass.  Order-preserving key of a finite fp16 bit pattern: keys compare as unsigned integers
// the way the values compare as numbers (-0 directly below +0).
__device__ inline unsigned f16_key(unsigned b) { return (b & 0x8000u) ? (~b & 0xffffu) : (b | 0x8000u); }
__device__ inline unsigned key_f16(unsigned k)
{
    const unsigned b = (k & 0x8000u) ? (k & 0x7fffu) : (~k & 0xffffu);
    return (b & 0x7fffu) ? b : 0u;  // a zero is reported as +0
}

// u(x) = round-half-even(254 x / D) for D > 0.  254 x and D are exact in double, the division is correctly
// rounded, and a quotient that is not a tie lies at least 2^-50 (relative) from the nearest half-integer,
// so rint() of the double quotient is the exact answer.  |u| <= 254 * 2^11.
__device__ __forceinline__ int zp_u(unsigned short xb, double D)
{
    return (int)__builtin_rint(254.0 * (double)f16_bits_to_float(xb) / D);
}

// The same u(x) without a division per element: with rD = the correctly rounded reciprocal of D (one
// division per vector, by the caller), q = a rD is within an ulp of a / D (a = 254 x, exact), the fused
// multiply-add gives the remainder a - q D exactly, and q + r rD rounds to the correctly rounded quotient
// (Markstein's correction step; its one exception, a divisor whose significand is all ones, cannot occur:
// D is a difference of two fp16 values and has at most 41 significant bits).  rint() then sees the same
// double as in zp_u.
__device__ __forceinline__ int zp_u_rcp(unsigned short xb, double D, double rD)
{
    const double a = 254.0 * (double)f16_bits_to_float(xb);
    const double q = a * rD;
    const double r = __builtin_fma(-q, D, a);
    return (int)__builtin_rint(__builtin_fma(r, rD, q));
}

// The record of a vector from the keys of its smallest and largest element: fp16 bits of lo and hi,
// zp = u(lo) + 127 (Eq. 2), and a zero for the sum of the codes, which the quantizer accumulates.
__device__ inline int4 make_const(unsigned kmin, unsigned kmax)
{
    const unsigned lo = key_f16(kmin), hi = key_f16(kmax);
    const double D = zp_range(lo | (hi << 16));
    int4 r;
    r.x = (int)(lo | (hi << 16));
    r.y = D > 0.0 ? zp_u((unsigned short)lo, D) + 127 : 0;
    r.z = 0;
    r.w = 0;
    return r;
}

// fp16( q * c_w / 127 ) for an int8 code q and a column constant given as fp16 bits, rounded once to nearest
// even: a weight rebuilt from its code (the variant that keeps no 16-bit weights).
// The exact quotient in 32-bit integer arithmetic: c_w = m * 2^E with an 11-bit m, so the value is
// (|q| * m / 127) * 2^E.  |q| * m (18 bits) is shifted up until its leading one sits at bit 30, which leaves
// the quotient by 127 with 24 or 25 significant bits, more than the 11 + 1 the rounding looks at; the
// division keeps its remainder as a sticky bit.  (Checked against 64-bit arithmetic for every code and every
// finite constant.)
__device__ inline unsigned short dequant_bits(int q, unsigned cwb)
{
    cwb &= 0x7fffu;
    if (q == 0 || cwb == 0) return 0;
    const unsigned sign = q < 0 ? 0x8000u : 0u;
    const unsigned a = (unsigned)(q < 0 ? -q : q);
    const unsigned e = cwb >> 10, f = cwb & 0x3ffu;
    const unsigned m = e ? 1024u + f : f;
    const int E = e ? (int)e - 25 : -24;
    const unsigned t = a * m;
    const int sh0 = __builtin_clz(t) - 1;
    const unsigned tn = t << sh0;                  // value = tn / 127 * 2^(E - sh0)
    const unsigned Q = tn / 127u, R = tn % 127u;
    const int msb = 31 - __builtin_clz(Q);         // 23 or 24
    int ev = msb + E - sh0;                        // value in [2^ev, 2^(ev+1))
    const bool normal = ev >= -14;
    const int sh = normal ? msb - 10 : sh0 - E - 24;  // Q / 2^sh counts fp16 quanta (2^(ev-10), or 2^-24 for subnormals); 13 .. 30
    unsigned mant = Q >> sh;
    const unsigned rem = Q & ((1u << sh) - 1u), half = 1u << (sh - 1);
    if (rem > half || (rem == half && (R != 0 || (mant & 1u)))) mant++;
    unsigned bits;
    if (normal) {
        if (mant == 2048) {
            mant = 1024;
            ev++;
        }
        bits = ((unsigned)(ev + 15) << 10) | (mant - 1024);
    } else {
        bits = mant;  // 1024 here is the smallest normal number, as it should be
    }
    return (unsigned short)(sign | bits);
}

// Smallest magnitude bit pattern whose value is >= alpha (0 if alpha <= 0,
// 0x7c00 if no finite fp16 reaches alpha).
__host__ inline unsigned threshold_bits(float alpha)
{
    if (!(alpha > 0.0f)) return 0u;            // alpha <= 0 (or NaN): every column qualifies
    if (alpha > 65504.0f) return 0x7c00u;      // above the largest finite fp16
    // binary search over the 0x7c00 non-negative finite patterns
    unsigned lo = 0, hi = 0x7bff;              // invariant: value(hi) >= alpha
    while (lo < hi) {
        unsigned mid = (lo + hi) / 2;
        unsigned e = mid >> 10, f = mid & 0x3ff;
        float v = e ? __builtin_ldexpf((float)(1024 + f), (int)e - 25) : __builtin_ldexpf((float)f, -24);
        if (v >= alpha) hi = mid; else lo = mid + 1;
    }
    return lo;
}

// ---- launchers (host side, defined next to their kernels) -------------------
// All return a hipError_t from hipGetLastError() after the launches.

// Column lists of the outlier scans (see prepass.hip), carved from the caller's workspace.
constexpr int MAXLISTS = 1024;  // runs of 256 columns; h <= LLMINT8_MAX_H needs 521
struct OutlierLists {
    int* count;               // [MAXLISTS] qualifying columns in each run of 256 columns
    int* cand;                // [lists][capc] their indices, ascending
    unsigned short* rowpart;  // [2][ceil(h / 512)][32] short-X scan only: partial row maxima (absmax), or the keys of
                              // the partial row minima followed by those of the maxima (zeropoint)
};
__host__ __device__ inline int list_capacity(int cap) { return cap < 256 ? cap : 256; }
inline size_t outlier_lists_bytes(int h, int cap)
{
    const size_t nl = (size_t)(h + 255) / 256, nwg = (size_t)(h + 511) / 512;
    return MAXLISTS * 4 + nl * list_capacity(cap) * 4 + 2 * nwg * 32 * 2;
}
inline OutlierLists carve_outlier_lists(char* base, int h, int cap)
{
    const size_t nl = (size_t)(h + 255) / 256;
    OutlierLists L;
    L.count = (int*)base;
    L.cand = (int*)(base + MAXLISTS * 4);
    L.rowpart = (unsigned short*)(base + MAXLISTS * 4 + nl * list_capacity(cap) * 4);
    return L;
}

// Positions of the lists in the overall order.  Call with all 256 threads of a workgroup; s_cnt and
// s_base are LDS arrays of MAXLISTS ints.  Returns the total number of qualifying columns.
__device__ inline int scan_lists(const int* __restrict__ count, int nl, int* s_cnt, int* s_base)
{
    __shared__ int s_wsum[4];
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    int c[4], sum = 0;
#pragma unroll
    for (int q = 0; q < 4; q++) {
        const int l = 4 * tid + q;
        c[q] = l < nl ? count[l] : 0;
        sum += c[q];
    }
    int incl = sum;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        const int t = __shfl_up(incl, d);
        if (lane >= d) incl += t;
    }
    __syncthreads();  // s_wsum may still be read by a previous call
    if (lane == 63) s_wsum[w] = incl;
    __syncthreads();
    int woff = 0, total = 0;
#pragma unroll
    for (int q = 0; q < 4; q++) {
        if (q < w) woff += s_wsum[q];
        total += s_wsum[q];
    }
    int run = woff + incl - sum;
#pragma unroll
    for (int q = 0; q < 4; q++) {
        const int l = 4 * tid + q;
        if (l < nl) {
            s_cnt[l] = c[q];
            s_base[l] = run;
        }
        run += c[q];
    }
    __syncthreads();
    return total;
}

// partial column maxima of an fp16 matrix M[rows][cols]: part[slab][cols] (u16 magnitude bits)
int colmax_slabs(int rows, int cols);
hipError_t launch_colmax_partial(const void* M, int rows, int cols, unsigned short* part, int nslab,
                                 hipStream_t st);
// slab maxima -> column lists; lists -> idx, count, status
hipError_t launch_outlier_lists(const unsigned short* part, int nslab, int h, unsigned thr, OutlierLists L, int cap,
                                hipStream_t st);
hipError_t launch_merge_lists(OutlierLists L, int h, int32_t* idx, int cap, int32_t* count, int32_t* status,
                              hipStream_t st);
// empty lists without a scan (no outlier columns: alpha = +inf)
hipError_t launch_clear_lists(OutlierLists L, int h, hipStream_t st);
// c[0 .. n) <- max(c): one constant for a whole tensor (shared_cx below does this to c_x)
hipError_t launch_spread_max(unsigned short* c, int n, hipStream_t st);
// row constants + codes + gathered columns fed by the lists; also writes idx, count, status
hipError_t launch_quantize_rows_lists(const void* X, int s, int h, OutlierLists L, int32_t* idx, int32_t* count,
                                      int32_t* status, int cap, int8_t* Xq, unsigned short* cx, unsigned short* Xo,
                                      int shared_cx, hipStream_t st);
// column scan of X that also leaves rowpart[ceil(h / 512)][s], the partial row maxima below the threshold
// (needs h % 8 == 0 and 16-byte aligned X, part), and the row constants + codes + gathered columns from them
hipError_t launch_colmax_rowmax(const void* X, int s, int h, unsigned short* part, int nslab, unsigned short* rowpart,
                                unsigned thr, hipStream_t st);
hipError_t launch_quantize_rows_rowpart(const void* X, int s, int h, OutlierLists L, unsigned thr,
                                        const unsigned short* rowpart, int32_t* idx, int32_t* count, int32_t* status,
                                        int cap, int8_t* Xq, unsigned short* cx, unsigned short* Xo, hipStream_t st);
// whole pre-pass of a short X (s <= 32): outlier scan, row constants, codes, gathered columns.
// zc != NULL: zeropoint records [s] in place of cx (which is then not written), codes u(x) - zp.
// With a column job the second kernel gets pitch / 256 more workgroups that do, from the column lists, what
// would otherwise take a kernel of its own before the matmul kernel: zeropoint: the per-column factors of
// launch_zp_kcol (pitch = zp_col_pitch(o)); absmax: the outlier rows of W rebuilt from the codes as
// launch_dequant_rows writes them (pitch = o rounded up to 256).
constexpr int JOB_MAX_CAP = 256;  // a column job is taken for outlier buffers up to this size (the set sits in LDS)
struct ColumnJob {
    const int8_t* Wq;    // tiled W_i8
    const void* wconst;  // zeropoint: [o] records of the columns of W; absmax: [o] c_w, fp16 bits
    void* out;           // zeropoint: three planes of pitch doubles; absmax: [opad][o] fp16
    int o, pitch;        // pitch 0: no job
};
hipError_t launch_prepass_small(const void* X, int s, int h, unsigned thr, OutlierLists L, int32_t* idx, int cap,
                                int32_t* count, int32_t* status, unsigned short* cx, unsigned short* Xo, int8_t* Xq,
                                int shared_cx, hipStream_t st, int4* zc = nullptr, const ColumnJob* cj = nullptr);
hipError_t launch_colmax_final(const unsigned short* part, int nslab, int cols, unsigned short* out,
                               hipStream_t st);
hipError_t launch_quantize_weight(const void* W, int h, int o, const unsigned short* cw, int8_t* Wq,
                                  hipStream_t st);
hipError_t launch_quantize_rows(const void* X, int s, int h, const int32_t* idx, const int32_t* count, int cap,
                                int8_t* Xq, unsigned short* cx, unsigned short* Xo, int shared_cx, hipStream_t st);
hipError_t launch_export_tiled(const int8_t* T, int rows, int h, int8_t* out, int ld_rows_major,
                               hipStream_t st);
// ---- zeropoint variant (Eq. 1-5; zeropoint.hip) ----
// Constants of one row of X / one column of W: {lo | hi << 16 (fp16 bits), zp, sum of the codes, 0}.
// part: scratch for 2 * zp_colrange_slabs(h, o) * o fp16 keys.
int zp_colrange_slabs(int h, int o);
hipError_t launch_zp_quantize_weight(const void* W, int h, int o, int8_t* Wq, int4* zc, unsigned short* part,
                                     hipStream_t st);
hipError_t launch_zp_quantize_rows(const void* X, int s, int h, const int32_t* idx, const int32_t* count, int cap,
                                   int8_t* Xq, int4* zc, unsigned short* Xo, hipStream_t st);
hipError_t launch_zp_quantize_rows_lists(const void* X, int s, int h, OutlierLists L, int32_t* idx, int32_t* count,
                                         int32_t* status, int cap, int8_t* Xq, int4* zc, unsigned short* Xo,
                                         const ColumnJob* cj, hipStream_t st);
// colc: three planes of zp_col_pitch(o) doubles (see zp_kcol_kernel).  The pitch covers every column a
// tile grid can touch (tiles are at most 256 columns wide), so the epilogues read it unguarded.
__host__ __device__ inline int zp_col_pitch(int o) { return ((o + 255) & ~255) + 256; }
hipError_t launch_zp_kcol(const int8_t* Wq, const int4* zcw, int h, int o, const int32_t* idx, const int32_t* count,
                          int cap, double* colc, hipStream_t st);
// What the GEMM epilogues need in place of c_x / c_w: T = C + zp_w[j] rowsum[i] + zp_x[i] K[j] (Eq. 5),
// Out = T D_x[i] D_w[j] / 254^2 + outlier product.  zcx NULL: absmax constants.
struct ZpArgs {
    const int4* zcx;     // [s] records of the rows of X
    const double* colc;  // per-column factors from launch_zp_kcol
    int pitch;           // zp_col_pitch(o)
};

// Wf: the original fp16 weights [h x o] (rows_are_slots = 0: outlier slot t uses row idx[t]), or the
// rebuilt rows [opad x o] of launch_dequant_rows (rows_are_slots = 1: slot t uses row t)
hipError_t launch_gemm_prefill(const int8_t* Xq, const unsigned short* cx, const unsigned short* Xo,
                               const int32_t* count, int cap, const int8_t* Wq, const unsigned short* cw,
                               const unsigned short* Wf, int rows_are_slots, const int32_t* idx, int s, int h, int o,
                               unsigned short* Out, int32_t* Cdbg, hipStream_t st, const ZpArgs* zp = nullptr);
// token counts that the weight-streaming kernel takes (the others go to the tiled kernel)
bool decode_kernel_takes(int s, int h, int o, bool zeropoint);
hipError_t launch_gemm_decode(const int8_t* Xq, const unsigned short* cx, const unsigned short* Xo,
                              const int32_t* count, int cap, const int8_t* Wq, const unsigned short* cw,
                              const unsigned short* Wf, int rows_are_slots, const int32_t* idx, int s, int h, int o,
                              unsigned short* Out, int32_t* Cdbg, hipStream_t st, const ZpArgs* zp = nullptr);
hipError_t launch_dequant_rows(const int8_t* Wq, const unsigned short* cw, int h, int o, const int32_t* idx,
                               const int32_t* count, int cap, unsigned short* Wo, hipStream_t st);

// tile shape the prefill GEMM chooses for a product of s x h by h x o (host arithmetic only)
int pick_cfg(int s, int h, int o);
// tile shape of the prefill GEMM forced by llmint8_debug_prefill_tile (-1: chosen from the shape)
extern std::atomic<int> g_force_cfg;
// work split of the decode kernel forced by llmint8_debug_decode_shape (-1: default)
extern std::atomic<int> g_decode_cfg;
// One-time set-up of the prefill kernels on the current device (dynamic LDS limit of every instantiation);
// returns the device's number of compute units.  Thread-safe; cheap after the first call on a device.
hipError_t prefill_device_setup(int* compute_units);

}  // namespace llmint8
