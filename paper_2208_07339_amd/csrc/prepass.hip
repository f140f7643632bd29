// Bandwidth-bound passes around the int8 GEMM: column absmax / outlier scan
// (Section 3.2), per-row absmax quantization of the non-outlier part of X and
// per-column absmax quantization of W (Sections 2.1, 3.1), layout export.
#include "common.h"

namespace llmint8 {

typedef unsigned short us8 __attribute__((ext_vector_type(8)));
typedef unsigned int u4 __attribute__((ext_vector_type(4)));
typedef unsigned int u2 __attribute__((ext_vector_type(2)));

// round-half-even of the exact quotient 127 x / c for fp16 x, c with |x| <= c,
// c > 0: 127 x is exact in fp32, the IEEE fp32 division is correctly rounded
// and a non-tie quotient lies further from a half-integer than half an fp32 ulp,
// so rint() of the fp32 quotient is the exact answer.  Do not replace the
// division by a multiplication with a reciprocal.
__device__ __forceinline__ int q8(float x, float c)
{
    return (int)__builtin_rintf((x * 127.0f) / c);
}

// ---------------------------------------------------------------------------
// Column maxima of |M[r][c]| over a slab of rows.  One workgroup covers 512
// columns (a wave reads 1 KiB of a row per load) and `rows_per_slab` rows, its
// four waves taking every fourth row.
// ---------------------------------------------------------------------------
__global__ void __launch_bounds__(256) colmax_partial_kernel(const unsigned short* __restrict__ M, int rows,
                                                             int cols, unsigned short* __restrict__ part,
                                                             int rows_per_slab, int vec_ok)
{
    __shared__ us8 red[4][64];
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    const int c0 = blockIdx.x * 512 + lane * 8;
    const int r0 = blockIdx.y * rows_per_slab;
    const int r1 = min(rows, r0 + rows_per_slab);
    us8 m = (us8)(0);
    if (vec_ok) {
        if (c0 < cols) {
            const unsigned short* p = M + (size_t)c0;
            int r = r0 + w;
            for (; r + 12 < r1; r += 16) {
                us8 a = *(const us8*)(p + (size_t)r * cols);
                us8 b = *(const us8*)(p + (size_t)(r + 4) * cols);
                us8 c = *(const us8*)(p + (size_t)(r + 8) * cols);
                us8 d = *(const us8*)(p + (size_t)(r + 12) * cols);
                a = __builtin_elementwise_max(a & (unsigned short)0x7fff, b & (unsigned short)0x7fff);
                c = __builtin_elementwise_max(c & (unsigned short)0x7fff, d & (unsigned short)0x7fff);
                m = __builtin_elementwise_max(m, __builtin_elementwise_max(a, c));
            }
            for (; r < r1; r += 4) {
                us8 a = *(const us8*)(p + (size_t)r * cols);
                m = __builtin_elementwise_max(m, a & (unsigned short)0x7fff);
            }
        }
    } else {
        for (int r = r0 + w; r < r1; r += 4)
#pragma unroll
            for (int e = 0; e < 8; e++)
                if (c0 + e < cols) {
                    unsigned short v = M[(size_t)r * cols + c0 + e] & 0x7fff;
                    m[e] = v > m[e] ? v : m[e];
                }
    }
    red[w][lane] = m;
    __syncthreads();
    if (w == 0) {
        m = __builtin_elementwise_max(__builtin_elementwise_max(red[0][lane], red[1][lane]),
                                      __builtin_elementwise_max(red[2][lane], red[3][lane]));
        unsigned short* o = part + (size_t)blockIdx.y * cols + c0;
        if (vec_ok) {
            if (c0 < cols) *(us8*)o = m;
        } else {
#pragma unroll
            for (int e = 0; e < 8; e++)
                if (c0 + e < cols) o[e] = m[e];
        }
    }
}

int colmax_slabs(int rows, int cols)
{
    // enough workgroups to cover the chip several times, at least 16 rows per slab
    int colblocks = (cols + 511) / 512;
    int want = (2048 + colblocks - 1) / colblocks;
    int maxslab = (rows + 15) / 16;
    int n = want < maxslab ? want : maxslab;
    if (n > 64) n = 64;
    if (n < 1) n = 1;
    return n;
}

static inline bool aligned16(const void* p) { return ((uintptr_t)p & 15) == 0; }

hipError_t launch_colmax_partial(const void* M, int rows, int cols, unsigned short* part, int nslab,
                                 hipStream_t st)
{
    int rps = (rows + nslab - 1) / nslab;
    int vec_ok = (cols % 8 == 0) && aligned16(M) && aligned16(part);
    dim3 grid((cols + 511) / 512, nslab);
    colmax_partial_kernel<<<grid, 256, 0, st>>>((const unsigned short*)M, rows, cols, part, rps, vec_ok);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------
// Reduce the slabs, apply the threshold, and write the qualifying column
// indices in ascending order.  One workgroup: flags are collected as wave
// ballots per 1024-column chunk, then a prefix sum over the ballots gives
// every set bit its position.
// ---------------------------------------------------------------------------
constexpr int CT = 1024;

__global__ void __launch_bounds__(CT) outlier_compact_kernel(const unsigned short* __restrict__ part, int nslab,
                                                             int h, unsigned thr, int32_t* __restrict__ idx,
                                                             int cap, int32_t* __restrict__ count,
                                                             int32_t* __restrict__ status)
{
    extern __shared__ unsigned long long ballots[];  // [nchunk * 16], then int bases[nchunk * 16]
    __shared__ int wtot[16];
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const int nchunk = (h + CT - 1) / CT;
    const int nent = nchunk * 16;
    int* bases = (int*)(ballots + nent);
    for (int c = 0; c < nchunk; c++) {
        const int j = c * CT + tid;
        unsigned m = 0;
        if (j < h)
            for (int sl = 0; sl < nslab; sl++) {
                unsigned v = part[(size_t)sl * h + j];
                m = v > m ? v : m;
            }
        const bool f = (j < h) && (m >= thr);
        unsigned long long b = __ballot(f);
        if (lane == 0) ballots[c * 16 + w] = b;
    }
    __syncthreads();
    const int per = (nent + CT - 1) / CT;
    const int e0 = tid * per;
    int mine = 0;
    for (int q = 0; q < per; q++)
        if (e0 + q < nent) mine += __popcll(ballots[e0 + q]);
    int incl = mine;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        int t = __shfl_up(incl, d);
        if (lane >= d) incl += t;
    }
    if (lane == 63) wtot[w] = incl;
    __syncthreads();
    int woff = 0, total = 0;
#pragma unroll
    for (int q = 0; q < 16; q++) {
        if (q < w) woff += wtot[q];
        total += wtot[q];
    }
    int run = woff + incl - mine;
    for (int q = 0; q < per; q++)
        if (e0 + q < nent) {
            bases[e0 + q] = run;
            run += __popcll(ballots[e0 + q]);
        }
    __syncthreads();
    for (int c = 0; c < nchunk; c++) {
        unsigned long long b = ballots[c * 16 + w];
        if ((b >> lane) & 1ull) {
            int pos = bases[c * 16 + w] + __popcll(b & ((1ull << lane) - 1ull));
            if (pos < cap) idx[pos] = c * CT + tid;
        }
    }
    if (tid == 0) {
        *count = total < cap ? total : cap;
        if (status) *status = total > cap ? 1 : 0;
    }
}

hipError_t launch_outlier_compact(const unsigned short* part, int nslab, int h, unsigned thr, int32_t* idx,
                                  int cap, int32_t* count, int32_t* status, hipStream_t st)
{
    int nchunk = (h + CT - 1) / CT;
    size_t shm = (size_t)nchunk * 16 * (sizeof(unsigned long long) + sizeof(int));
    outlier_compact_kernel<<<1, CT, shm, st>>>(part, nslab, h, thr, idx, cap, count, status);
    return hipGetLastError();
}

// out[c] = max over slabs (weights: this is c_w as fp16 bits)
__global__ void __launch_bounds__(256) colmax_final_kernel(const unsigned short* __restrict__ part, int nslab,
                                                           int cols, unsigned short* __restrict__ out)
{
    int j = blockIdx.x * 256 + threadIdx.x;
    if (j >= cols) return;
    unsigned m = 0;
    for (int sl = 0; sl < nslab; sl++) {
        unsigned v = part[(size_t)sl * cols + j];
        m = v > m ? v : m;
    }
    out[j] = (unsigned short)m;
}

hipError_t launch_colmax_final(const unsigned short* part, int nslab, int cols, unsigned short* out,
                               hipStream_t st)
{
    colmax_final_kernel<<<(cols + 255) / 256, 256, 0, st>>>(part, nslab, cols, out);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------
// W_i8 in the tiled layout (tile rows = output columns, tile K = features).
// One workgroup: 32 features (one kt) x 256 output columns (8 tiles), staged
// through LDS so that the transposed tiles leave as whole 1 KiB pieces.
// ---------------------------------------------------------------------------
__global__ void __launch_bounds__(256) quantize_weight_kernel(const unsigned short* __restrict__ W, int h, int o,
                                                              const unsigned short* __restrict__ cw,
                                                              int8_t* __restrict__ Wq, int KT, int JT, int vec_ok)
{
    __shared__ __attribute__((aligned(16))) int8_t stage[8 * TILE_BYTES];
    const int tid = threadIdx.x;
    const int kt = blockIdx.y;
    const int jt0 = blockIdx.x * 8;
    const int cg = tid & 31, sub = tid >> 5;
    const int j0 = jt0 * 32 + cg * 8;
    float c[8];
#pragma unroll
    for (int e = 0; e < 8; e++) c[e] = (j0 + e < o) ? f16_bits_to_float(cw[j0 + e]) : 0.0f;
#pragma unroll
    for (int q = 0; q < 4; q++) {
        const int kk = q * 8 + sub;
        const int k = kt * 32 + kk;
        us8 v = (us8)(0);
        if (k < h) {
            if (vec_ok && j0 + 8 <= o) {
                v = *(const us8*)(W + (size_t)k * o + j0);
            } else {
#pragma unroll
                for (int e = 0; e < 8; e++)
                    if (j0 + e < o) v[e] = W[(size_t)k * o + j0 + e];
            }
        }
#pragma unroll
        for (int e = 0; e < 8; e++) {
            int qv = (c[e] > 0.0f) ? q8(f16_bits_to_float(v[e]), c[e]) : 0;
            const int jj = cg * 8 + e;
            stage[(jj >> 5) * TILE_BYTES + tile_byte(jj & 31, kk)] = (int8_t)qv;
        }
    }
    __syncthreads();
    const int tile = tid >> 5;
    if (jt0 + tile < JT) {
        const u4* src = (const u4*)(stage + tid * 32);
        u4* dst = (u4*)(Wq + ((size_t)(jt0 + tile) * KT + kt) * TILE_BYTES + (tid & 31) * 32);
        dst[0] = src[0];
        dst[1] = src[1];
    }
}

hipError_t launch_quantize_weight(const void* W, int h, int o, const unsigned short* cw, int8_t* Wq,
                                  hipStream_t st)
{
    const int KT = k_tiles(h), JT = row_tiles(o);
    int vec_ok = (o % 8 == 0) && aligned16(W);
    dim3 grid((JT + 7) / 8, KT);
    quantize_weight_kernel<<<grid, 256, 0, st>>>((const unsigned short*)W, h, o, cw, Wq, KT, JT, vec_ok);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------
// Row constants over the non-outlier columns, and the gathered outlier
// columns Xo.  One workgroup per row; the outlier set is a bitmap in LDS.
// ---------------------------------------------------------------------------
__global__ void __launch_bounds__(256) row_absmax_kernel(const unsigned short* __restrict__ X, int s, int h,
                                                         const int32_t* __restrict__ idx,
                                                         const int32_t* __restrict__ count, int cap, int opad,
                                                         unsigned short* __restrict__ cx,
                                                         unsigned short* __restrict__ Xo, int vec_ok)
{
    extern __shared__ unsigned bitmap[];  // ceil(h / 32) words, then 4 words of reduction space
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const int nw = (h + 31) / 32;
    unsigned* red = bitmap + nw;
    int cnt = *count;
    cnt = cnt < 0 ? 0 : (cnt > cap ? cap : cnt);
    for (int q = tid; q < nw; q += 256) bitmap[q] = 0;
    __syncthreads();
    for (int t = tid; t < cnt; t += 256) {
        unsigned j = (unsigned)idx[t];
        if (j < (unsigned)h) atomicOr(&bitmap[j >> 5], 1u << (j & 31));
    }
    __syncthreads();
    const int i = blockIdx.x;
    const unsigned short* row = X + (size_t)i * h;
    unsigned m = 0;
    if (vec_ok) {
        for (int c0 = tid * 8; c0 < h; c0 += 2048) {
            us8 v = *(const us8*)(row + c0) & (unsigned short)0x7fff;
            unsigned bits = (bitmap[c0 >> 5] >> (c0 & 31)) & 0xffu;
#pragma unroll
            for (int e = 0; e < 8; e++) {
                unsigned x = ((bits >> e) & 1u) ? 0u : (unsigned)v[e];
                m = x > m ? x : m;
            }
        }
    } else {
        for (int c = tid; c < h; c += 256) {
            unsigned x = ((bitmap[c >> 5] >> (c & 31)) & 1u) ? 0u : (unsigned)(row[c] & 0x7fff);
            m = x > m ? x : m;
        }
    }
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) {
        unsigned t = (unsigned)__shfl_xor((int)m, d);
        m = t > m ? t : m;
    }
    if (lane == 0) red[w] = m;
    __syncthreads();
    if (tid == 0) {
        unsigned a = red[0] > red[1] ? red[0] : red[1];
        unsigned b = red[2] > red[3] ? red[2] : red[3];
        cx[i] = (unsigned short)(a > b ? a : b);
    }
    for (int t = tid; t < opad; t += 256) {
        unsigned short v = 0;
        if (t < cnt) {
            unsigned j = (unsigned)idx[t];
            if (j < (unsigned)h) v = row[j];
        }
        Xo[(size_t)i * opad + t] = v;
    }
}

// ---------------------------------------------------------------------------
// X_i8 in the tiled layout.  One workgroup: 32 rows (one row tile) x 256
// features (8 tiles, contiguous in the output).  Rows are read as 512-byte
// pieces, coded, scattered into LDS at their tile position and written out as
// one contiguous 8 KiB run.
// ---------------------------------------------------------------------------
__global__ void __launch_bounds__(256) quantize_rows_kernel(const unsigned short* __restrict__ X, int s, int h,
                                                            const int32_t* __restrict__ idx,
                                                            const int32_t* __restrict__ count, int cap,
                                                            const unsigned short* __restrict__ cx,
                                                            int8_t* __restrict__ Xq, int KT, int vec_ok)
{
    __shared__ __attribute__((aligned(16))) int8_t stage[8 * TILE_BYTES];
    __shared__ unsigned bitmap[8];
    const int tid = threadIdx.x;
    const int rt = blockIdx.x;
    const int k0 = blockIdx.y * 256;
    int cnt = *count;
    cnt = cnt < 0 ? 0 : (cnt > cap ? cap : cnt);
    if (tid < 8) bitmap[tid] = 0;
    __syncthreads();
    for (int t = tid; t < cnt; t += 256) {
        unsigned j = (unsigned)idx[t] - (unsigned)k0;
        if (j < 256u) atomicOr(&bitmap[j >> 5], 1u << (j & 31));
    }
    __syncthreads();
    const int kseg = (tid & 31) * 8;
    const int k = k0 + kseg;
    const unsigned bits = (bitmap[kseg >> 5] >> (kseg & 31)) & 0xffu;
#pragma unroll
    for (int q = 0; q < 4; q++) {
        const int r = q * 8 + (tid >> 5);
        const int i = rt * 32 + r;
        us8 v = (us8)(0);
        float c = 0.0f;
        if (i < s) {
            c = f16_bits_to_float(cx[i]);
            const unsigned short* row = X + (size_t)i * h;
            if (vec_ok && k + 8 <= h) {
                v = *(const us8*)(row + k);
            } else {
#pragma unroll
                for (int e = 0; e < 8; e++)
                    if (k + e < h) v[e] = row[k + e];
            }
        }
        unsigned lo = 0, hi = 0;
#pragma unroll
        for (int e = 0; e < 8; e++) {
            int qv = (c > 0.0f && !((bits >> e) & 1u)) ? q8(f16_bits_to_float(v[e]), c) : 0;
            unsigned byte = (unsigned)qv & 0xffu;
            if (e < 4) lo |= byte << (8 * e); else hi |= byte << (8 * (e - 4));
        }
        u2 pk = {lo, hi};
        *(u2*)(stage + (kseg >> 5) * TILE_BYTES + tile_byte(r, kseg & 31)) = pk;
    }
    __syncthreads();
    const int kt0 = k0 >> 5;
#pragma unroll
    for (int half = 0; half < 2; half++) {
        const int off = half * 4096 + tid * 16;
        if (kt0 + (off >> 10) < KT)
            *(u4*)(Xq + ((size_t)rt * KT + kt0) * TILE_BYTES + off) = *(const u4*)(stage + off);
    }
}

hipError_t launch_quantize_rows(const void* X, int s, int h, const int32_t* idx, const int32_t* count, int cap,
                                int8_t* Xq, unsigned short* cx, unsigned short* Xo, hipStream_t st)
{
    const int KT = k_tiles(h), RT = row_tiles(s);
    const int opad = opad_of(cap);
    int vec_ok = (h % 8 == 0) && aligned16(X);
    size_t shm = ((size_t)(h + 31) / 32 + 4) * sizeof(unsigned);
    row_absmax_kernel<<<s, 256, shm, st>>>((const unsigned short*)X, s, h, idx, count, cap, opad, cx, Xo, vec_ok);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    dim3 grid(RT, (KT * 32 + 255) / 256);
    quantize_rows_kernel<<<grid, 256, 0, st>>>((const unsigned short*)X, s, h, idx, count, cap, cx, Xq, KT, vec_ok);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------
// Tiled int8 -> plain matrix.  Element (r, k) of the tiled matrix goes to
// out[r * sr + k * sk].  One thread per 16-byte lane chunk.  Support code.
// ---------------------------------------------------------------------------
__global__ void __launch_bounds__(256) export_tiled_kernel(const int8_t* __restrict__ T, int rows, int h, int KT,
                                                           int8_t* __restrict__ out, size_t sr, size_t sk,
                                                           size_t nchunks)
{
    size_t g = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (g >= nchunks) return;
    const size_t tile = g >> 6;
    const int l = (int)(g & 63);
    const int rt = (int)(tile / KT), kt = (int)(tile % KT);
    const int r = rt * 32 + (l & 31);
    const int kb = kt * 32 + (l >> 5) * 16;
    if (r >= rows) return;
    u4 v = *(const u4*)(T + g * 16);
    const int8_t* b = (const int8_t*)&v;
#pragma unroll
    for (int e = 0; e < 16; e++)
        if (kb + e < h) out[(size_t)r * sr + (size_t)(kb + e) * sk] = b[e];
}

hipError_t launch_export_tiled(const int8_t* T, int rows, int h, int8_t* out, int rows_major, hipStream_t st)
{
    const int KT = k_tiles(h), RT = row_tiles(rows);
    size_t nchunks = (size_t)RT * KT * 64;
    size_t sr = rows_major ? (size_t)h : 1, sk = rows_major ? 1 : (size_t)rows;
    export_tiled_kernel<<<(unsigned)((nchunks + 255) / 256), 256, 0, st>>>(T, rows, h, KT, out, sr, sk, nchunks);
    return hipGetLastError();
}

}  // namespace llmint8
