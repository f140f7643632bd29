// Bandwidth-bound passes around the int8 GEMM: column absmax / outlier scan
// (Section 3.2), per-row absmax quantization of the non-outlier part of X and
// per-column absmax quantization of W (Sections 2.1, 3.1), layout export.
#include "common.h"

namespace llmint8 {

typedef unsigned short us8 __attribute__((ext_vector_type(8)));
typedef unsigned int u4 __attribute__((ext_vector_type(4)));
typedef unsigned int u2 __attribute__((ext_vector_type(2)));

// round-half-even of the exact quotient 127 x / c for fp16 x, c with |x| <= c, c > 0.
// a = 127 x is exact in fp32; a non-tie quotient a / c lies further from a half-integer than half an
// fp32 ulp, so rint() of the correctly rounded fp32 quotient is the exact answer.  The correctly
// rounded quotient comes without a division per element: with rc = the correctly rounded reciprocal of
// c (one IEEE division per row / column, by the caller), q = a rc is within an ulp of a / c, the fused
// multiply-add gives the remainder r = a - q c exactly, and q + r rc rounds to the correctly rounded
// quotient (Markstein's correction step).  Checked against integer arithmetic for every pair of fp16
// values |x| <= c.  Do not drop the correction step, and do not let rc be an approximate reciprocal.
__device__ __forceinline__ int q8(float x, float c, float rc)
{
    const float a = x * 127.0f;
    const float q = a * rc;
    const float r = __builtin_fmaf(-q, c, a);
    return (int)__builtin_rintf(__builtin_fmaf(r, rc, q));
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
// The same column scan for X (vector path only) that also prepares the row
// constants: rowpart[colblock][row] = largest magnitude BELOW the threshold
// among the row's entries in this workgroup's 512 columns.  Entries of
// non-outlier columns are all below the threshold, so the maximum of a row's
// partials is its constant c_x unless that maximum sits in an outlier column
// (row_const_kernel checks this once the outlier columns are known).
// ---------------------------------------------------------------------------
typedef unsigned short us2 __attribute__((ext_vector_type(2)));

__device__ __forceinline__ unsigned short hmax8(us8 v)
{
    us2 a = __builtin_elementwise_max(__builtin_elementwise_max(v.s01, v.s23), __builtin_elementwise_max(v.s45, v.s67));
    return a.x > a.y ? a.x : a.y;
}

__global__ void __launch_bounds__(256) colmax_rowmax_kernel(const unsigned short* __restrict__ M, int rows, int cols,
                                                            unsigned short* __restrict__ part,
                                                            unsigned short* __restrict__ rowpart, int rows_per_slab,
                                                            unsigned thr)
{
    __shared__ us8 red[4][64];
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    const int c0 = blockIdx.x * 512 + lane * 8;
    const int r0 = blockIdx.y * rows_per_slab;
    const int r1 = min(rows, r0 + rows_per_slab);
    const bool in = c0 < cols;
    const unsigned short* p = M + (size_t)(in ? c0 : 0);
    const us8 thrv = (us8)((unsigned short)thr);
    us8 m = (us8)(0);
    // Unconditional loads, so that all four of a pass are in flight together (a row past the slab repeats its last
    // one: the maxima do not change, its row maximum is not stored), and the next pass's four are requested before
    // this pass's reductions.
    us8 nv[4];
    auto request = [&](int r) {
#pragma unroll
        for (int u = 0; u < 4; u++) {
            const int rr = r + 4 * u < r1 ? r + 4 * u : r1 - 1;
            nv[u] = *(const us8*)(p + (size_t)rr * cols);
        }
    };
    if (r0 + w < r1) request(r0 + w);
    for (int r = r0 + w; r < r1; r += 16) {
        us8 v[4];
        unsigned short x[4];
#pragma unroll
        for (int u = 0; u < 4; u++) v[u] = nv[u];
        request(r + 16);
#pragma unroll
        for (int u = 0; u < 4; u++) {
            v[u] = in ? v[u] & (unsigned short)0x7fff : (us8)(0);  // lanes past the last column read column 0
            m = __builtin_elementwise_max(m, v[u]);
            const us8 below = v[u] & __builtin_convertvector(v[u] < thrv, us8);  // lanes that reach the threshold drop out
            x[u] = hmax8(below);
        }
        // two rows per register through the cross-lane reduction
        us2 a = {x[0], x[1]}, b = {x[2], x[3]};
#pragma unroll
        for (int d = 32; d >= 1; d >>= 1) {
            const us2 ta = __builtin_bit_cast(us2, __shfl_xor(__builtin_bit_cast(int, a), d));
            const us2 tb = __builtin_bit_cast(us2, __shfl_xor(__builtin_bit_cast(int, b), d));
            a = __builtin_elementwise_max(a, ta);
            b = __builtin_elementwise_max(b, tb);
        }
        if (lane == 0) {
            unsigned short* o = rowpart + (size_t)blockIdx.x * rows;
            if (r < r1) o[r] = a.x;
            if (r + 4 < r1) o[r + 4] = a.y;
            if (r + 8 < r1) o[r + 8] = b.x;
            if (r + 12 < r1) o[r + 12] = b.y;
        }
    }
    red[w][lane] = m;
    __syncthreads();
    if (w == 0 && in) {
        m = __builtin_elementwise_max(__builtin_elementwise_max(red[0][lane], red[1][lane]),
                                      __builtin_elementwise_max(red[2][lane], red[3][lane]));
        *(us8*)(part + (size_t)blockIdx.y * cols + c0) = m;
    }
}

hipError_t launch_colmax_rowmax(const void* X, int s, int h, unsigned short* part, int nslab, unsigned short* rowpart,
                                unsigned thr, hipStream_t st)
{
    const int rps = (s + nslab - 1) / nslab;
    dim3 grid((h + 511) / 512, nslab);
    colmax_rowmax_kernel<<<grid, 256, 0, st>>>((const unsigned short*)X, s, h, part, rowpart, rps, thr);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------
// Outlier column lists.  The scan kernels cut the h columns into runs of 256;
// run l gets the list cand[l][0 .. capc) of its columns whose maximum reaches
// the threshold, ascending, and count[l] = how many there are (capc =
// min(cap, 256); a longer list can only happen when |O| > cap anyway).  The
// outlier set is the concatenation of the lists, cut off after cap entries.
// Kernels that need it (row constants, quantizer) read the lists themselves:
// scan_lists() gives every list its position in the overall order.
// ---------------------------------------------------------------------------

// One workgroup = 256 columns x 4 groups of slabs: reduce the slab maxima, apply the threshold, list.
__global__ void __launch_bounds__(1024) outlier_lists_kernel(const unsigned short* __restrict__ part, int nslab,
                                                             int h, unsigned thr, OutlierLists L, int capc)
{
    __shared__ unsigned short red[4][256];
    __shared__ int wcnt[4];
    const int tid = threadIdx.x, lane = tid & 63;
    const int c = tid & 255, g = tid >> 8;
    const int j = blockIdx.x * 256 + c;
    unsigned m = 0;
    if (j < h)
        for (int sl = g; sl < nslab; sl += 32) {  // 8 independent loads in flight
            unsigned v[8];
#pragma unroll
            for (int u = 0; u < 8; u++) {
                const int q = sl + 4 * u;
                v[u] = q < nslab ? (unsigned)part[(size_t)q * h + j] : 0u;
            }
#pragma unroll
            for (int u = 0; u < 8; u++) m = v[u] > m ? v[u] : m;
        }
    red[g][c] = (unsigned short)m;
    __syncthreads();
    bool f = false;
    if (g == 0) {
        const unsigned a = red[0][c] > red[1][c] ? red[0][c] : red[1][c];
        const unsigned b = red[2][c] > red[3][c] ? red[2][c] : red[3][c];
        f = (j < h) && ((a > b ? a : b) >= thr);
    }
    const unsigned long long bal = __ballot(f);
    if (g == 0 && lane == 0) wcnt[tid >> 6] = __popcll(bal);
    __syncthreads();
    if (g == 0) {
        const int w = tid >> 6;
        int woff = 0, total = 0;
#pragma unroll
        for (int q = 0; q < 4; q++) {
            if (q < w) woff += wcnt[q];
            total += wcnt[q];
        }
        if (f) {
            const int pos = woff + __popcll(bal & ((1ull << lane) - 1ull));
            if (pos < capc) L.cand[(size_t)blockIdx.x * capc + pos] = j;
        }
        if (tid == 0) L.count[blockIdx.x] = total;
    }
}

hipError_t launch_outlier_lists(const unsigned short* part, int nslab, int h, unsigned thr, OutlierLists L, int cap,
                                hipStream_t st)
{
    outlier_lists_kernel<<<(h + 255) / 256, 1024, 0, st>>>(part, nslab, h, thr, L, list_capacity(cap));
    return hipGetLastError();
}

// (scan_lists(), the positions of the lists in the overall order, lives in common.h: zeropoint.hip uses it too)

// idx, count, status from the lists (the stand-alone outlier scan ends with this)
__global__ void __launch_bounds__(256) merge_lists_kernel(OutlierLists L, int nl, int capc, int32_t* __restrict__ idx,
                                                          int cap, int32_t* __restrict__ count,
                                                          int32_t* __restrict__ status)
{
    __shared__ int s_cnt[MAXLISTS], s_base[MAXLISTS];
    const int tid = threadIdx.x;
    const int total = scan_lists(L.count, nl, s_cnt, s_base);
    for (int b = tid; b < nl; b += 256) {
        const int n = s_cnt[b] < capc ? s_cnt[b] : capc;
        const int base = s_base[b];
        for (int e = 0; e < n && base + e < cap; e++) idx[base + e] = L.cand[(size_t)b * capc + e];
    }
    if (tid == 0) {
        *count = total < cap ? total : cap;
        if (status) *status = total > cap ? 1 : 0;
    }
}

hipError_t launch_merge_lists(OutlierLists L, int h, int32_t* idx, int cap, int32_t* count, int32_t* status,
                              hipStream_t st)
{
    merge_lists_kernel<<<1, 256, 0, st>>>(L, (h + 255) / 256, list_capacity(cap), idx, cap, count, status);
    return hipGetLastError();
}

// no outlier columns at all (alpha = +inf is known on the host): empty lists without a scan of X
__global__ void __launch_bounds__(256) clear_lists_kernel(int* __restrict__ count, int nl)
{
    const int l = blockIdx.x * 256 + threadIdx.x;
    if (l < nl) count[l] = 0;
}

hipError_t launch_clear_lists(OutlierLists L, int h, hipStream_t st)
{
    const int nl = (h + 255) / 256;
    clear_lists_kernel<<<(nl + 255) / 256, 256, 0, st>>>(L.count, nl);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------
// One constant for a whole tensor (absmax quantization as Section 2.1 defines
// it; the row-wise and tensor-wise baselines of Table 1): every entry of
// c[0 .. n) is replaced by the largest of them.  One workgroup; n is s or o.
// ---------------------------------------------------------------------------
__global__ void __launch_bounds__(1024) spread_max_kernel(unsigned short* __restrict__ c, int n)
{
    __shared__ unsigned red[16];
    const int tid = threadIdx.x;
    unsigned m = 0;
    for (int q = tid; q < n; q += 1024) {
        const unsigned v = c[q];
        m = v > m ? v : m;
    }
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) {
        const unsigned t = (unsigned)__shfl_xor((int)m, d);
        m = t > m ? t : m;
    }
    if ((tid & 63) == 0) red[tid >> 6] = m;
    __syncthreads();  // every read of c is done before the first write below
#pragma unroll
    for (int q = 0; q < 16; q++) m = red[q] > m ? red[q] : m;
    for (int q = tid; q < n; q += 1024) c[q] = (unsigned short)m;
}

hipError_t launch_spread_max(unsigned short* c, int n, hipStream_t st)
{
    spread_max_kernel<<<1, 1024, 0, st>>>(c, n);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------
// Short X (s <= 32 tokens), two kernels for the whole pre-pass.
//
// scan_small_kernel: a workgroup owns 512 columns (two lists) and sees all s
// rows of them, so it knows which of its columns are outliers and can take
// every row's maximum over the rest of its columns: rowpart[wg][32].
//
// quantize_small_kernel: every workgroup (256 features of the one row tile)
// places the lists, reduces the partial row maxima to the row constants and
// quantizes its features; workgroup 0 also writes idx, count, status, c_x and
// the gathered columns Xo.
//
// ZP: zeropoint constants (Section 2.1, Eq. 1-3) in place of absmax ones.  The
// scan leaves, per row, the keys of the smallest and the largest entry among
// its non-outlier columns and clears the rows' records; the quantizer turns
// them into the records (range, zeropoint), writes the codes u(x) - zp and adds
// its part of every row's sum of codes into the record.
// ---------------------------------------------------------------------------
template <bool ZP>
__global__ void __launch_bounds__(256) scan_small_kernel(const unsigned short* __restrict__ X, int s, int h,
                                                         unsigned thr, int vec_ok, OutlierLists L, int capc,
                                                         int4* __restrict__ zc)
{
    __shared__ us8 red[4][64];
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const int c0 = blockIdx.x * 512 + lane * 8;
    us8 v[8];
    us8 m = (us8)(0);
    if (vec_ok) {
        // unconditional loads (a row or column that does not exist: row 0 / column 0 again, zeroed afterwards), so
        // that all eight are in flight together: each under its own bounds check was waited for before the next
        // was issued, eight round trips to memory in a row
#pragma unroll
        for (int r = 0; r < 8; r++) {
            const int i = w + 4 * r;
            v[r] = *(const us8*)(X + (size_t)(i < s ? i : 0) * h + (c0 < h ? c0 : 0));
        }
#pragma unroll
        for (int r = 0; r < 8; r++)
            if (!(w + 4 * r < s && c0 < h)) v[r] = (us8)(0);
    } else {
#pragma unroll
        for (int r = 0; r < 8; r++) {
            const int i = w + 4 * r;
            v[r] = (us8)(0);
            if (i < s && c0 < h) {
                const unsigned short* p = X + (size_t)i * h + c0;
#pragma unroll
                for (int e = 0; e < 8; e++)
                    if (c0 + e < h) v[r][e] = p[e];
            }
        }
    }
#pragma unroll
    for (int r = 0; r < 8; r++) {
        if (!ZP) v[r] &= (unsigned short)0x7fff;
        m = __builtin_elementwise_max(m, v[r] & (unsigned short)0x7fff);
    }
    if (ZP && blockIdx.x == 0 && tid < s) zc[tid] = make_int4(0, 0, 0, 0);
    red[w][lane] = m;
    __syncthreads();
    m = __builtin_elementwise_max(__builtin_elementwise_max(red[0][lane], red[1][lane]),
                                  __builtin_elementwise_max(red[2][lane], red[3][lane]));
    unsigned flags = 0;
#pragma unroll
    for (int e = 0; e < 8; e++)
        if (c0 + e < h && (unsigned)m[e] >= thr) flags |= 1u << e;
    // partial row maxima over this workgroup's non-outlier columns
#pragma unroll
    for (int r = 0; r < 8; r++) {
        if constexpr (!ZP) {
            unsigned mx = 0;
#pragma unroll
            for (int e = 0; e < 8; e++) {
                const unsigned x = ((flags >> e) & 1u) ? 0u : (unsigned)v[r][e];
                mx = x > mx ? x : mx;
            }
#pragma unroll
            for (int d = 32; d >= 1; d >>= 1) {
                const unsigned t = (unsigned)__shfl_xor((int)mx, d);
                mx = t > mx ? t : mx;
            }
            if (lane == 0) L.rowpart[(size_t)blockIdx.x * 32 + w + 4 * r] = (unsigned short)mx;  // 0 for rows >= s
        } else {
            // keys of the smallest and the largest entry; an empty set (rows >= s, nothing but outlier
            // columns) is min 0xffff above max 0
            unsigned kmin = 0xffffu, kmax = 0u;
            if (w + 4 * r < s) {
#pragma unroll
                for (int e = 0; e < 8; e++)
                    if (!((flags >> e) & 1u) && c0 + e < h) {
                        const unsigned k = f16_key(v[r][e]);
                        kmin = k < kmin ? k : kmin;
                        kmax = k > kmax ? k : kmax;
                    }
            }
#pragma unroll
            for (int d = 32; d >= 1; d >>= 1) {
                const unsigned a = (unsigned)__shfl_xor((int)kmin, d), b = (unsigned)__shfl_xor((int)kmax, d);
                kmin = a < kmin ? a : kmin;
                kmax = b > kmax ? b : kmax;
            }
            if (lane == 0) {
                L.rowpart[(size_t)blockIdx.x * 32 + w + 4 * r] = (unsigned short)kmin;
                L.rowpart[((size_t)gridDim.x + blockIdx.x) * 32 + w + 4 * r] = (unsigned short)kmax;
            }
        }
    }
    if (w == 0) {  // the two lists of this workgroup (lanes 0-31, lanes 32-63), ascending: lane, then bit
        const int mine = __popc(flags);
        int incl = mine;
#pragma unroll
        for (int d = 1; d < 64; d <<= 1) {
            const int t = __shfl_up(incl, d);
            if (lane >= d) incl += t;
        }
        const int low = __shfl(incl, 31), all = __shfl(incl, 63);
        const int list = blockIdx.x * 2 + (lane >> 5);
        int pos = incl - mine - (lane >= 32 ? low : 0);
#pragma unroll
        for (int e = 0; e < 8; e++)
            if ((flags >> e) & 1u) {
                if (pos < capc) L.cand[(size_t)list * capc + pos] = c0 + e;
                pos++;
            }
        if (lane == 0) L.count[list] = low;
        if (lane == 32 && blockIdx.x * 512 + 256 < h) L.count[list] = all - low;
    }
}

template <bool ZP>
__global__ void __launch_bounds__(256) quantize_small_kernel(const unsigned short* __restrict__ X, int s, int h,
                                                             OutlierLists L, int capc, int vec_ok,
                                                             int32_t* __restrict__ idx, int cap, int opad,
                                                             int32_t* __restrict__ count,
                                                             int32_t* __restrict__ status,
                                                             unsigned short* __restrict__ cx,
                                                             unsigned short* __restrict__ Xo,
                                                             int8_t* __restrict__ Xq, int KT, int shared_cx,
                                                             int4* __restrict__ zc, ColumnJob cj)
{
    extern __shared__ unsigned fullmap[];  // ceil(h / 32) words, used only when |O| > cap
    __shared__ __attribute__((aligned(16))) int8_t stage[8 * TILE_BYTES];
    __shared__ int s_cnt[MAXLISTS], s_base[MAXLISTS];
    __shared__ unsigned s_part[8][32];
    __shared__ unsigned s_cxb[32];
    __shared__ unsigned s_part_lo[ZP ? 8 : 1][32];  // zeropoint: s_part / s_cxb hold the keys of the maxima, these of the minima
    __shared__ unsigned s_lo[ZP ? 32 : 1];
    __shared__ double s_D[ZP ? 32 : 1], s_rD[ZP ? 32 : 1];  // zeropoint: range of each row and its reciprocal
    __shared__ int s_z[ZP ? 32 : 1];                        // and its zeropoint
    __shared__ unsigned bitmap[8];
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const int k0 = blockIdx.x * 256;
    const int nl = (h + 255) / 256, nwg = (h + 511) / 512;

    // One-call paths: the workgroups past those of the quantizer take a column job (see ColumnJob).  They read
    // the outlier set straight from the lists (slot t of the set is entry t of their concatenation) into LDS
    // first, so that a thread's loads of its column's codes in those rows do not wait for one another.
    const int nquant = (KT * 32 + 255) / 256;
    if ((int)blockIdx.x >= nquant) {
        __shared__ int s_idx[JOB_MAX_CAP];
        const int total = scan_lists(L.count, nl, s_cnt, s_base);
        const int cnt = total < cap ? total : cap;  // cap <= JOB_MAX_CAP (checked by the launcher)
        __syncthreads();
        for (int b = tid; b < nl; b += 256) {
            const int n = s_cnt[b] < capc ? s_cnt[b] : capc;
            for (int e = 0; e < n && s_base[b] + e < cap; e++) s_idx[s_base[b] + e] = L.cand[(size_t)b * capc + e];
        }
        __syncthreads();
        const int j = ((int)blockIdx.x - nquant) * 256 + tid;
        if (j >= cj.pitch) return;
        const int8_t* col = cj.Wq + (size_t)(j >> 5) * KT * TILE_BYTES;  // column j of W: row j & 31 of these tiles
        // codes of column j in outlier rows t0 .. t0+7 (0 and not valid where there is none)
        auto codes8 = [&](int t0, int* q, bool* ok) {
#pragma unroll
            for (int u = 0; u < 8; u++) {
                const unsigned k = (t0 + u < cnt) ? (unsigned)s_idx[t0 + u] : 0xffffffffu;
                ok[u] = k < (unsigned)h;
                q[u] = ok[u] ? col[(size_t)(k >> 5) * TILE_BYTES + tile_byte(j & 31, (int)(k & 31))] : 0;
            }
        };
        if constexpr (ZP) {
            // the per-column factors of Eq. 5, as zp_kcol_kernel makes them from idx / count: p = D_w / 254,
            // q = zp_w p, r = K p, K = (sum of the column's codes outside the outlier rows) + (h - |O|) zp_w;
            // zero for the padding columns j >= o
            double p = 0.0, q = 0.0, r = 0.0;
            if (j < cj.o) {
                const int4 rec = ((const int4*)cj.wconst)[j];
                long long sum = rec.z;
                int used = 0;
                for (int t0 = 0; t0 < cnt; t0 += 8) {
                    int c8[8];
                    bool ok[8];
                    codes8(t0, c8, ok);
#pragma unroll
                    for (int u = 0; u < 8; u++) {
                        sum -= c8[u];
                        used += ok[u] ? 1 : 0;
                    }
                }
                p = zp_range((unsigned)rec.x) * (1.0 / 254.0);
                q = (double)rec.y * p;
                r = (double)(sum + (long long)(h - used) * rec.y) * p;
            }
            double* colc = (double*)cj.out;
            colc[j] = p;
            colc[(size_t)cj.pitch + j] = q;
            colc[2 * (size_t)cj.pitch + j] = r;
        } else {
            // the outlier rows of W rebuilt from the codes, as dequant_rows_kernel writes them: slot t holds
            // row idx[t], zeros from |O| to opad
            if (j >= cj.o) return;
            const unsigned cwb = ((const unsigned short*)cj.wconst)[j];
            unsigned short* Wo = (unsigned short*)cj.out;
            for (int t0 = 0; t0 < cnt; t0 += 8) {
                int c8[8];
                bool ok[8];
                codes8(t0, c8, ok);
#pragma unroll
                for (int u = 0; u < 8; u++)
                    if (t0 + u < cnt)  // the same for every thread: no arithmetic for the empty slots
                        Wo[(size_t)(t0 + u) * cj.o + j] = ok[u] ? dequant_bits(c8[u], cwb) : (unsigned short)0;
            }
            for (int t = cnt; t < opad; t++) Wo[(size_t)t * cj.o + j] = 0;
        }
        return;
    }

    // Everything whose address is known is requested first, so that the latencies overlap: this
    // thread's 8 features of 4 rows, and its share of the partial row maxima.
    const int kseg = (tid & 31) * 8;
    const int k = k0 + kseg;
    us8 xv[4];
    if (vec_ok && k + 8 <= h) {
        // unconditional (a row that does not exist: row 0 again; its codes come out as 0 because its constant
        // is 0), or the compiler waits for each load before it issues the next
#pragma unroll
        for (int q = 0; q < 4; q++) {
            const int r = q * 8 + (tid >> 5);
            xv[q] = *(const us8*)(X + (size_t)(r < s ? r : 0) * h + k);
        }
    } else {
#pragma unroll
        for (int q = 0; q < 4; q++) {
            const int r = q * 8 + (tid >> 5);
            xv[q] = (us8)(0);
            if (r < s) {
                const unsigned short* row = X + (size_t)r * h;
#pragma unroll
                for (int e = 0; e < 8; e++)
                    if (k + e < h) xv[q][e] = row[k + e];
            }
        }
    }
    unsigned rp_max = 0;  // max over workgroups gq, gq+8, .. of rowpart[.][i]
    unsigned rp_min = 0xffffu;
    {
        const int i = tid & 31, gq = tid >> 5;
        for (int b = gq; b < nwg; b += 32) {  // 4 independent loads in flight
            unsigned t4[4], t5[4];
#pragma unroll
            for (int u = 0; u < 4; u++) {
                const size_t at = (size_t)(b + 8 * u) * 32 + i;
                if constexpr (ZP) {
                    t5[u] = (b + 8 * u < nwg) ? (unsigned)L.rowpart[at] : 0xffffu;
                    t4[u] = (b + 8 * u < nwg) ? (unsigned)L.rowpart[(size_t)nwg * 32 + at] : 0u;
                } else {
                    t4[u] = (b + 8 * u < nwg) ? (unsigned)L.rowpart[at] : 0u;
                }
            }
#pragma unroll
            for (int u = 0; u < 4; u++) {
                rp_max = t4[u] > rp_max ? t4[u] : rp_max;
                if constexpr (ZP) rp_min = t5[u] < rp_min ? t5[u] : rp_min;
            }
        }
    }

    if (tid < 8) bitmap[tid] = 0;
    const int total = scan_lists(L.count, nl, s_cnt, s_base);
    const int cnt = total < cap ? total : cap;
    const bool overflow = total > cap;

    // ---- row constants
    if (!overflow) {
        s_part[tid >> 5][tid & 31] = rp_max;
        if constexpr (ZP) s_part_lo[tid >> 5][tid & 31] = rp_min;
        __syncthreads();
        if (tid < 32) {
            unsigned m2 = 0, m1 = 0xffffu;
#pragma unroll
            for (int q = 0; q < 8; q++) {
                m2 = s_part[q][tid] > m2 ? s_part[q][tid] : m2;
                if constexpr (ZP) m1 = s_part_lo[q][tid] < m1 ? s_part_lo[q][tid] : m1;
            }
            s_cxb[tid] = m2;
            if constexpr (ZP) s_lo[tid] = m1;
        }
    } else {
        // only the first cap columns count as outliers: redo the row maxima with their bitmap
        const int nw = (h + 31) / 32;
        for (int q = tid; q < nw; q += 256) fullmap[q] = 0;
        __syncthreads();
        for (int b = tid; b < nl; b += 256) {
            const int n = s_cnt[b] < capc ? s_cnt[b] : capc;
            for (int e = 0; e < n && s_base[b] + e < cap; e++) {
                const unsigned j = (unsigned)L.cand[(size_t)b * capc + e];
                atomicOr(&fullmap[j >> 5], 1u << (j & 31));
            }
        }
        __syncthreads();
        for (int i = w; i < 32; i += 4) {
            unsigned mx = 0, mn = 0xffffu;
            if (i < s)
                for (int c = lane; c < h; c += 64) {
                    if constexpr (ZP) {
                        if (!((fullmap[c >> 5] >> (c & 31)) & 1u)) {
                            const unsigned k = f16_key(X[(size_t)i * h + c]);
                            mn = k < mn ? k : mn;
                            mx = k > mx ? k : mx;
                        }
                    } else {
                        const unsigned x =
                            ((fullmap[c >> 5] >> (c & 31)) & 1u) ? 0u : (unsigned)(X[(size_t)i * h + c] & 0x7fff);
                        mx = x > mx ? x : mx;
                    }
                }
#pragma unroll
            for (int d = 32; d >= 1; d >>= 1) {
                const unsigned t = (unsigned)__shfl_xor((int)mx, d);
                mx = t > mx ? t : mx;
                if constexpr (ZP) {
                    const unsigned u = (unsigned)__shfl_xor((int)mn, d);
                    mn = u < mn ? u : mn;
                }
            }
            if (lane == 0) {
                s_cxb[i] = mx;
                if constexpr (ZP) s_lo[i] = mn;
            }
        }
    }
    // ---- outlier columns among this workgroup's 256 features: list k0 / 256
    {
        const int b = k0 >> 8;
        const int n = s_cnt[b] < capc ? s_cnt[b] : capc;
        for (int e = tid; e < n; e += 256)
            if (s_base[b] + e < cap) {
                const unsigned j = (unsigned)L.cand[(size_t)b * capc + e] - (unsigned)k0;
                if (j < 256u) atomicOr(&bitmap[j >> 5], 1u << (j & 31));
            }
    }
    __syncthreads();
    if constexpr (ZP) {  // the rows' records: range, zeropoint (a row with no non-outlier column: all zero)
        if (tid < 32) {
            int4 r = make_int4(0, 0, 0, 0);
            if (tid < s && s_lo[tid] <= s_cxb[tid]) r = make_const(s_lo[tid], s_cxb[tid]);
            const double D = zp_range((unsigned)r.x);
            s_D[tid] = D;
            s_rD[tid] = D > 0.0 ? 1.0 / D : 0.0;
            s_z[tid] = r.y;
            if (blockIdx.x == 0 && tid < s) {  // the sum of the codes (word 2) was cleared by the scan and is added to below
                int* rec = (int*)(zc + tid);
                rec[0] = r.x;
                rec[1] = r.y;
            }
        }
        __syncthreads();
    }
    if (!ZP && shared_cx) {  // tensor-wise baseline: one constant, the largest of the row maxima (rows >= s hold 0)
        unsigned t = 0;
#pragma unroll
        for (int q = 0; q < 32; q++) t = s_cxb[q] > t ? s_cxb[q] : t;
        __syncthreads();
        if (tid < 32) s_cxb[tid] = t;
        __syncthreads();
    }

    // ---- workgroup 0: the outputs of the outlier scan, c_x, Xo
    if (blockIdx.x == 0) {
        for (int b = tid; b < nl; b += 256) {
            const int n = s_cnt[b] < capc ? s_cnt[b] : capc;
            const int base = s_base[b];
            for (int e = 0; e < n && base + e < cap; e++) idx[base + e] = L.cand[(size_t)b * capc + e];
        }
        __syncthreads();  // idx is read back by other threads of this workgroup
        for (int q = tid; q < s * opad; q += 256) {
            const int i = q / opad, t = q - i * opad;
            Xo[q] = t < cnt ? X[(size_t)i * h + idx[t]] : (unsigned short)0;
        }
        if (tid == 0) {
            *count = cnt;
            if (status) *status = overflow ? 1 : 0;
        }
        if (!ZP && tid < s) cx[tid] = (unsigned short)s_cxb[tid];
    }

    // ---- codes of 32 rows x 256 features into the tiled layout
    const unsigned bits = (bitmap[kseg >> 5] >> (kseg & 31)) & 0xffu;
#pragma unroll
    for (int q = 0; q < 4; q++) {
        const int r = q * 8 + (tid >> 5);
        const us8 v = xv[q];
        unsigned lo = 0, hi = 0;
        if constexpr (ZP) {
            const double D = (r < s) ? s_D[r] : 0.0, rD = s_rD[r];
            const int z = s_z[r];
            int part = 0;
#pragma unroll
            for (int e = 0; e < 8; e++) {
                int qv = 0;
                if (D > 0.0 && k + e < h && !((bits >> e) & 1u)) qv = zp_u_rcp(v[e], D, rD) - z;
                part += qv;
                const unsigned byte = (unsigned)qv & 0xffu;
                if (e < 4) lo |= byte << (8 * e); else hi |= byte << (8 * (e - 4));
            }
            // the 32 lanes that share row r (one half of a wave) add up their parts
#pragma unroll
            for (int d = 16; d >= 1; d >>= 1) part += __shfl_xor(part, d);
            if ((tid & 31) == 0 && r < s && part) atomicAdd(&zc[r].z, part);
        } else {
            const float c = (r < s) ? f16_bits_to_float((unsigned short)s_cxb[r]) : 0.0f;
            const float rc = c > 0.0f ? 1.0f / c : 0.0f;
#pragma unroll
            for (int e = 0; e < 8; e++) {
                const int qv = (c > 0.0f && !((bits >> e) & 1u)) ? q8(f16_bits_to_float(v[e]), c, rc) : 0;
                const unsigned byte = (unsigned)qv & 0xffu;
                if (e < 4) lo |= byte << (8 * e); else hi |= byte << (8 * (e - 4));
            }
        }
        u2 pk = {lo, hi};
        *(u2*)(stage + (kseg >> 5) * TILE_BYTES + tile_byte(r, kseg & 31)) = pk;
    }
    __syncthreads();
    const int kt0 = k0 >> 5;
#pragma unroll
    for (int half = 0; half < 2; half++) {
        const int off = half * 4096 + tid * 16;
        if (kt0 + (off >> 10) < KT) *(u4*)(Xq + (size_t)kt0 * TILE_BYTES + off) = *(const u4*)(stage + off);
    }
}

hipError_t launch_prepass_small(const void* X, int s, int h, unsigned thr, OutlierLists L, int32_t* idx, int cap,
                                int32_t* count, int32_t* status, unsigned short* cx, unsigned short* Xo, int8_t* Xq,
                                int shared_cx, hipStream_t st, int4* zc, const ColumnJob* cj)
{
    const int capc = list_capacity(cap);
    const int vec_ok = (h % 8 == 0) && aligned16(X);
    const int KT = k_tiles(h);
    const int nscan = (h + 511) / 512, nquant = (KT * 32 + 255) / 256;
    const size_t shm = ((size_t)(h + 31) / 32) * sizeof(unsigned);
    const ColumnJob job = (cj && cap <= JOB_MAX_CAP) ? *cj : ColumnJob{nullptr, nullptr, nullptr, 0, 0};
    if (zc) {
        scan_small_kernel<true><<<nscan, 256, 0, st>>>((const unsigned short*)X, s, h, thr, vec_ok, L, capc, zc);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
        quantize_small_kernel<true><<<nquant + job.pitch / 256, 256, shm, st>>>(
            (const unsigned short*)X, s, h, L, capc, vec_ok, idx, cap, opad_of(cap), count, status, cx, Xo, Xq, KT, 0, zc,
            job);
        return hipGetLastError();
    }
    scan_small_kernel<false><<<nscan, 256, 0, st>>>((const unsigned short*)X, s, h, thr, vec_ok, L, capc, nullptr);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    quantize_small_kernel<false><<<nquant + job.pitch / 256, 256, shm, st>>>(
        (const unsigned short*)X, s, h, L, capc, vec_ok, idx, cap, opad_of(cap), count, status, cx, Xo, Xq, KT, shared_cx,
        nullptr, job);
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
    // The vector path requests its column constants and the four rows of W without conditions (a row past h: the
    // last one again, zeroed below), so that the loads are in flight together instead of one after the other.
    const bool vec = vec_ok && j0 + 8 <= o;
    us8 cv = (us8)(0), wv[4];
    if (vec) {
        cv = *(const us8*)(cw + j0);
#pragma unroll
        for (int q = 0; q < 4; q++) {
            const int k = kt * 32 + q * 8 + sub;
            wv[q] = *(const us8*)(W + (size_t)(k < h ? k : h - 1) * o + j0);
        }
    }
    float c[8], rc[8];
#pragma unroll
    for (int e = 0; e < 8; e++) {
        c[e] = vec ? f16_bits_to_float(cv[e]) : (j0 + e < o) ? f16_bits_to_float(cw[j0 + e]) : 0.0f;
        rc[e] = c[e] > 0.0f ? 1.0f / c[e] : 0.0f;
    }
#pragma unroll
    for (int q = 0; q < 4; q++) {
        const int kk = q * 8 + sub;
        const int k = kt * 32 + kk;
        us8 v = (us8)(0);
        if (k < h) {
            if (vec) {
                v = wv[q];
            } else {
#pragma unroll
                for (int e = 0; e < 8; e++)
                    if (j0 + e < o) v[e] = W[(size_t)k * o + j0 + e];
            }
        }
#pragma unroll
        for (int e = 0; e < 8; e++) {
            int qv = (c[e] > 0.0f) ? q8(f16_bits_to_float(v[e]), c[e], rc[e]) : 0;
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
    int vec_ok = (o % 8 == 0) && aligned16(W) && aligned16(cw);
    dim3 grid((JT + 7) / 8, KT);
    quantize_weight_kernel<<<grid, 256, 0, st>>>((const unsigned short*)W, h, o, cw, Wq, KT, JT, vec_ok);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------
// Row constants over the non-outlier columns, and the gathered outlier
// columns Xo.  One workgroup per row; the outlier set is a bitmap in LDS,
// built from idx / count, or (LISTS) straight from the column lists of the
// scan, in which case workgroup 0 also writes idx, count and status.
// ---------------------------------------------------------------------------
template <bool LISTS>
__global__ void __launch_bounds__(256) row_absmax_kernel(const unsigned short* __restrict__ X, int s, int h,
                                                         int32_t* __restrict__ idx, int32_t* __restrict__ count,
                                                         int32_t* __restrict__ status, OutlierLists L, int capc,
                                                         int cap, int opad, unsigned short* __restrict__ cx,
                                                         unsigned short* __restrict__ Xo, int vec_ok)
{
    extern __shared__ unsigned bitmap[];  // ceil(h / 32) words, then 4 words of reduction space
    __shared__ int s_cnt[LISTS ? MAXLISTS : 1], s_base[LISTS ? MAXLISTS : 1];
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const int nw = (h + 31) / 32;
    unsigned* red = bitmap + nw;
    const int i = blockIdx.x;
    const unsigned short* row = X + (size_t)i * h;
    int cnt;
    for (int q = tid; q < nw; q += 256) bitmap[q] = 0;
    if (LISTS) {
        const int nl = (h + 255) / 256;
        const int total = scan_lists(L.count, nl, s_cnt, s_base);  // its barriers also publish the cleared bitmap
        cnt = total < cap ? total : cap;
        for (int b = tid; b < nl; b += 256) {
            const int n = s_cnt[b] < capc ? s_cnt[b] : capc;
            const int base = s_base[b];
            for (int e = 0; e < n && base + e < cap; e++) {
                const int j = L.cand[(size_t)b * capc + e];
                atomicOr(&bitmap[j >> 5], 1u << (j & 31));
                Xo[(size_t)i * opad + base + e] = row[j];
                if (i == 0) idx[base + e] = j;
            }
        }
        for (int t = cnt + tid; t < opad; t += 256) Xo[(size_t)i * opad + t] = 0;
        if (i == 0 && tid == 0) {
            *count = cnt;
            if (status) *status = total > cap ? 1 : 0;
        }
    } else {
        cnt = *count;
        cnt = cnt < 0 ? 0 : (cnt > cap ? cap : cnt);
        __syncthreads();
        for (int t = tid; t < cnt; t += 256) {
            unsigned j = (unsigned)idx[t];
            if (j < (unsigned)h) atomicOr(&bitmap[j >> 5], 1u << (j & 31));
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
    __syncthreads();
    unsigned m = 0;
    if (vec_ok) {
        // four unconditional loads in flight per pass (past the row: its start again, skipped below)
        for (int c0 = tid * 8; c0 < h; c0 += 4 * 2048) {
            us8 v[4];
#pragma unroll
            for (int u = 0; u < 4; u++) {
                const int c = c0 + u * 2048;
                v[u] = *(const us8*)(row + (c < h ? c : 0)) & (unsigned short)0x7fff;
            }
#pragma unroll
            for (int u = 0; u < 4; u++) {
                const int c = c0 + u * 2048;
                if (c < h) {
                    const unsigned bits = (bitmap[c >> 5] >> (c & 31)) & 0xffu;
#pragma unroll
                    for (int e = 0; e < 8; e++) {
                        const unsigned x = ((bits >> e) & 1u) ? 0u : (unsigned)v[u][e];
                        m = x > m ? x : m;
                    }
                }
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
}

// ---------------------------------------------------------------------------
// Row constants from the partial row maxima of colmax_rowmax_kernel, one wave
// per row; also the gathered outlier columns Xo and (workgroup 0) idx, count,
// status, as row_absmax_kernel<true>.  With m1 = the largest below-threshold
// magnitude of the row and mo = the largest such magnitude inside the outlier
// columns: mo < m1 means m1 sits in a non-outlier column, so c_x = m1.
// Otherwise (rare), and whenever more columns qualify than cap allows (then
// the columns beyond cap count as ordinary ones and their large entries
// belong to c_x), the workgroup scans that row again without the outlier
// columns.  Needs h % 8 == 0 and a 16-byte aligned X.
// ---------------------------------------------------------------------------
constexpr int RC_SLOTS = 256;  // outlier columns kept in LDS; more: every row takes the slow path

__global__ void __launch_bounds__(256) row_const_kernel(const unsigned short* __restrict__ X, int s, int h,
                                                        OutlierLists L, int capc, int cap, int opad, unsigned thr,
                                                        const unsigned short* __restrict__ rowpart, int ncb,
                                                        int32_t* __restrict__ idx, int32_t* __restrict__ count,
                                                        int32_t* __restrict__ status, unsigned short* __restrict__ cx,
                                                        unsigned short* __restrict__ Xo)
{
    extern __shared__ unsigned fullmap[];  // ceil(h / 32) words, filled only when some row needs the slow path
    __shared__ int s_cnt[MAXLISTS], s_base[MAXLISTS];
    __shared__ int s_idx[RC_SLOTS];
    __shared__ int s_slow, s_again[4];
    __shared__ unsigned s_red[4];
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const int nl = (h + 255) / 256, nw = (h + 31) / 32;
    // this wave's row, and its first 128 partial maxima requested before anything else (they do not depend on
    // the lists; unconditional: a block or row that does not exist reads one that does and is skipped below)
    const int i = blockIdx.x * 4 + w;
    const unsigned short rp0 = rowpart[(size_t)(lane < ncb ? lane : 0) * s + (i < s ? i : 0)];
    const unsigned short rp1 = rowpart[(size_t)(lane + 64 < ncb ? lane + 64 : 0) * s + (i < s ? i : 0)];
    const int total = scan_lists(L.count, nl, s_cnt, s_base);
    const int cnt = total < cap ? total : cap;
    const bool all_slow = total > cap || cnt > RC_SLOTS;
    if (tid == 0) s_slow = all_slow ? 1 : 0;
    for (int b = tid; b < nl; b += 256) {
        const int n = s_cnt[b] < capc ? s_cnt[b] : capc;
        const int base = s_base[b];
        for (int e = 0; e < n && base + e < cap; e++) {
            const int j = L.cand[(size_t)b * capc + e];
            if (base + e < RC_SLOTS) s_idx[base + e] = j;
            if (blockIdx.x == 0) idx[base + e] = j;
        }
    }
    if (blockIdx.x == 0 && tid == 0) {
        *count = cnt;
        if (status) *status = total > cap ? 1 : 0;
    }
    __syncthreads();
    const unsigned short* row = X + (size_t)(i < s ? i : 0) * h;
    unsigned m1 = 0, mo = 0;
    bool need = false;
    if (i < s && !all_slow) {
        if (lane < ncb) m1 = rp0;
        if (lane + 64 < ncb && rp1 > m1) m1 = rp1;
        for (int cb = lane + 128; cb < ncb; cb += 64) {
            const unsigned v = rowpart[(size_t)cb * s + i];
            m1 = v > m1 ? v : m1;
        }
        for (int t = lane; t < opad; t += 64) {
            unsigned short v = 0;
            if (t < cnt) {
                v = row[s_idx[t]];
                const unsigned a = v & 0x7fffu;
                if (a < thr) mo = a > mo ? a : mo;
            }
            Xo[(size_t)i * opad + t] = v;
        }
#pragma unroll
        for (int d = 32; d >= 1; d >>= 1) {
            const unsigned t1 = (unsigned)__shfl_xor((int)m1, d), t2 = (unsigned)__shfl_xor((int)mo, d);
            m1 = t1 > m1 ? t1 : m1;
            mo = t2 > mo ? t2 : mo;
        }
        need = mo >= m1 && m1 > 0;
    }
    if (lane == 0) {
        s_again[w] = (i < s && (all_slow || need)) ? 1 : 0;
        if (need) s_slow = 1;
    }
    __syncthreads();
    if (s_slow) {  // uniform: the bitmap of all outlier columns, then the whole workgroup scans each such row again
        for (int q = tid; q < nw; q += 256) fullmap[q] = 0;
        __syncthreads();
        if (cnt <= RC_SLOTS) {  // the list is in LDS already
            for (int t2 = tid; t2 < cnt; t2 += 256) atomicOr(&fullmap[s_idx[t2] >> 5], 1u << (s_idx[t2] & 31));
        } else {
            for (int b = tid; b < nl; b += 256) {
                const int n = s_cnt[b] < capc ? s_cnt[b] : capc;
                const int base = s_base[b];
                for (int e = 0; e < n && base + e < cap; e++) {
                    const int j = L.cand[(size_t)b * capc + e];
                    atomicOr(&fullmap[j >> 5], 1u << (j & 31));
                }
            }
        }
        __syncthreads();
        for (int r4 = 0; r4 < 4; r4++) {
            if (!s_again[r4]) continue;  // uniform
            const int i2 = blockIdx.x * 4 + r4;
            const unsigned short* row2 = X + (size_t)i2 * h;
            unsigned m = 0;
            // h is a multiple of 8 here.  One slow row makes this workgroup the kernel's last, and every pass of
            // this loop is a round trip to memory of its own: twelve 16-byte loads in flight per lane take a row
            // of 49 152 features in two passes (24 in one pass are no faster and cost 65 more registers).  (With each load under its own bounds check the compiler waited
            // for every one of them in turn: 16 us for the kernel instead of 5 whenever one row came here.)
            constexpr int RU = 12;
            for (int c0 = tid * 8; c0 < h; c0 += RU * 2048) {
                us8 v[RU];
#pragma unroll
                for (int u = 0; u < RU; u++) {  // unconditional loads (past the row: its start again, unused below),
                    const int c = c0 + u * 2048;  // so that the compiler issues them together
                    v[u] = *(const us8*)(row2 + (c < h ? c : 0)) & (unsigned short)0x7fff;
                }
#pragma unroll
                for (int u = 0; u < RU; u++) {
                    const int c = c0 + u * 2048;
                    if (c < h) {
                        const unsigned bits = (fullmap[c >> 5] >> (c & 31)) & 0xffu;
#pragma unroll
                        for (int e = 0; e < 8; e++) {
                            const unsigned x = ((bits >> e) & 1u) ? 0u : (unsigned)v[u][e];
                            m = x > m ? x : m;
                        }
                    }
                }
            }
#pragma unroll
            for (int d = 32; d >= 1; d >>= 1) {
                const unsigned t = (unsigned)__shfl_xor((int)m, d);
                m = t > m ? t : m;
            }
            if (lane == 0) s_red[w] = m;
            __syncthreads();
            if (tid == 0) {
                const unsigned a = s_red[0] > s_red[1] ? s_red[0] : s_red[1];
                const unsigned b = s_red[2] > s_red[3] ? s_red[2] : s_red[3];
                cx[i2] = (unsigned short)(a > b ? a : b);
            }
            if (all_slow) {  // gather straight from the lists: the LDS copy may not hold them all
                for (int b = tid; b < nl; b += 256) {
                    const int n = s_cnt[b] < capc ? s_cnt[b] : capc;
                    const int base = s_base[b];
                    for (int e = 0; e < n && base + e < cap; e++)
                        Xo[(size_t)i2 * opad + base + e] = row2[L.cand[(size_t)b * capc + e]];
                }
                for (int t = cnt + tid; t < opad; t += 256) Xo[(size_t)i2 * opad + t] = 0;
            }
            __syncthreads();  // s_red is reused by the next row
        }
    }
    if (i < s && lane == 0 && !(all_slow || need)) cx[i] = (unsigned short)m1;
}

// ---------------------------------------------------------------------------
// X_i8 in the tiled layout.  One workgroup: 32 rows (one row tile) x 256
// features (8 tiles, contiguous in the output).  Rows are read as 512-byte
// pieces, coded, scattered into LDS at their tile position and written out as
// one contiguous 8 KiB run.
// ---------------------------------------------------------------------------
template <bool LISTS>
__global__ void __launch_bounds__(256) quantize_rows_kernel(const unsigned short* __restrict__ X, int s, int h,
                                                            const int32_t* __restrict__ idx,
                                                            const int32_t* __restrict__ count, OutlierLists L,
                                                            int capc, int cap, const unsigned short* __restrict__ cx,
                                                            int8_t* __restrict__ Xq, int KT, int vec_ok)
{
    __shared__ __attribute__((aligned(16))) int8_t stage[8 * TILE_BYTES];
    __shared__ unsigned bitmap[8];
    __shared__ int s_red[4];
    const int tid = threadIdx.x;
    const int rt = blockIdx.x;
    const int k0 = blockIdx.y * 256;
    const int kseg = (tid & 31) * 8;
    const int k = k0 + kseg;
    if (tid < 8) bitmap[tid] = 0;
    if (LISTS) {
        // the outlier columns among these 256 features are list k0 / 256; its position in the overall
        // order is the number of qualifying columns before it
        const int b = k0 >> 8;
        int before = 0;
        for (int l = tid; l < b; l += 256) before += L.count[l];
#pragma unroll
        for (int d = 32; d >= 1; d >>= 1) before += __shfl_xor(before, d);
        if ((tid & 63) == 0) s_red[tid >> 6] = before;
        __syncthreads();
        const int base = s_red[0] + s_red[1] + s_red[2] + s_red[3];
        const int n = L.count[b] < capc ? L.count[b] : capc;
        for (int e = tid; e < n; e += 256)
            if (base + e < cap) {
                const unsigned j = (unsigned)L.cand[(size_t)b * capc + e] - (unsigned)k0;
                if (j < 256u) atomicOr(&bitmap[j >> 5], 1u << (j & 31));
            }
    } else {
        int cnt = *count;
        cnt = cnt < 0 ? 0 : (cnt > cap ? cap : cnt);
        __syncthreads();
        for (int t = tid; t < cnt; t += 256) {
            unsigned j = (unsigned)idx[t] - (unsigned)k0;
            if (j < 256u) atomicOr(&bitmap[j >> 5], 1u << (j & 31));
        }
    }
    __syncthreads();
    const unsigned bits = (bitmap[kseg >> 5] >> (kseg & 31)) & 0xffu;
    // (requested here and not at the top of the kernel, in front of the look-up of this block's outlier columns:
    // measured, that order is slower, 12.7 against 12.1 us on a 4096 x 5120 X)
    // The loads of the thread's four rows first, all of them unconditional (a row past the last one: the last
    // one again, its constant taken as 0 below), so that they are in flight together: under a bounds check of
    // its own each was waited for before the next was issued, four round trips to memory in a row.
    us8 vq[4];
    float cq[4];
    const bool vec = vec_ok && k + 8 <= h;
#pragma unroll
    for (int q = 0; q < 4; q++) {
        const int i = rt * 32 + q * 8 + (tid >> 5);
        const int ii = i < s ? i : s - 1;
        cq[q] = f16_bits_to_float(cx[ii]);
        if (i >= s) cq[q] = 0.0f;
        vq[q] = (us8)(0);
        if (vec) vq[q] = *(const us8*)(X + (size_t)ii * h + k);
    }
#pragma unroll
    for (int q = 0; q < 4; q++) {
        const int r = q * 8 + (tid >> 5);
        const int i = rt * 32 + r;
        us8 v = vq[q];
        const float c = cq[q];
        if (!vec && i < s) {
            const unsigned short* row = X + (size_t)i * h;
#pragma unroll
            for (int e = 0; e < 8; e++)
                if (k + e < h) v[e] = row[k + e];
        }
        const float rc = c > 0.0f ? 1.0f / c : 0.0f;
        unsigned lo = 0, hi = 0;
#pragma unroll
        for (int e = 0; e < 8; e++) {
            int qv = (c > 0.0f && !((bits >> e) & 1u)) ? q8(f16_bits_to_float(v[e]), c, rc) : 0;
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
                                int8_t* Xq, unsigned short* cx, unsigned short* Xo, int shared_cx, hipStream_t st)
{
    const int KT = k_tiles(h), RT = row_tiles(s);
    const int opad = opad_of(cap);
    int vec_ok = (h % 8 == 0) && aligned16(X);
    size_t shm = ((size_t)(h + 31) / 32 + 4) * sizeof(unsigned);
    const OutlierLists none = {nullptr, nullptr, nullptr};
    row_absmax_kernel<false><<<s, 256, shm, st>>>((const unsigned short*)X, s, h, (int32_t*)idx, (int32_t*)count,
                                                  nullptr, none, 0, cap, opad, cx, Xo, vec_ok);
    hipError_t e = hipGetLastError();
    if (e == hipSuccess && shared_cx) e = launch_spread_max(cx, s, st);
    if (e != hipSuccess) return e;
    dim3 grid(RT, (KT * 32 + 255) / 256);
    quantize_rows_kernel<false><<<grid, 256, 0, st>>>((const unsigned short*)X, s, h, idx, count, none, 0, cap, cx, Xq,
                                                      KT, vec_ok);
    return hipGetLastError();
}

// the same two steps fed by the column lists of the scan; also writes idx, count, status
hipError_t launch_quantize_rows_lists(const void* X, int s, int h, OutlierLists L, int32_t* idx, int32_t* count,
                                      int32_t* status, int cap, int8_t* Xq, unsigned short* cx, unsigned short* Xo,
                                      int shared_cx, hipStream_t st)
{
    const int KT = k_tiles(h), RT = row_tiles(s);
    const int opad = opad_of(cap), capc = list_capacity(cap);
    int vec_ok = (h % 8 == 0) && aligned16(X);
    size_t shm = ((size_t)(h + 31) / 32 + 4) * sizeof(unsigned);
    row_absmax_kernel<true><<<s, 256, shm, st>>>((const unsigned short*)X, s, h, idx, count, status, L, capc, cap, opad,
                                                 cx, Xo, vec_ok);
    hipError_t e = hipGetLastError();
    if (e == hipSuccess && shared_cx) e = launch_spread_max(cx, s, st);
    if (e != hipSuccess) return e;
    dim3 grid(RT, (KT * 32 + 255) / 256);
    quantize_rows_kernel<true><<<grid, 256, 0, st>>>((const unsigned short*)X, s, h, idx, count, L, capc, cap, cx, Xq, KT,
                                                     vec_ok);
    return hipGetLastError();
}

// the per-call pre-pass for s > 32 when X allows 16-byte loads: row constants from the partial row maxima
// of the column scan instead of another full pass over X
hipError_t launch_quantize_rows_rowpart(const void* X, int s, int h, OutlierLists L, unsigned thr,
                                        const unsigned short* rowpart, int32_t* idx, int32_t* count, int32_t* status,
                                        int cap, int8_t* Xq, unsigned short* cx, unsigned short* Xo, hipStream_t st)
{
    const int KT = k_tiles(h), RT = row_tiles(s);
    const int opad = opad_of(cap), capc = list_capacity(cap);
    const size_t shm = ((size_t)(h + 31) / 32) * sizeof(unsigned);
    row_const_kernel<<<(s + 3) / 4, 256, shm, st>>>((const unsigned short*)X, s, h, L, capc, cap, opad, thr, rowpart,
                                                    (h + 511) / 512, idx, count, status, cx, Xo);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    dim3 grid(RT, (KT * 32 + 255) / 256);
    quantize_rows_kernel<true><<<grid, 256, 0, st>>>((const unsigned short*)X, s, h, idx, count, L, capc, cap, cx, Xq, KT,
                                                     1);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------
// Outlier rows of W rebuilt from the codes (variant that keeps no 16-bit
// weights): Wo[t][j] = fp16( W_i8[idx[t]][j] * c_w[j] / 127 ), one rounding
// to nearest even of the exact quotient, zero rows for t >= |O|.
// ---------------------------------------------------------------------------

__global__ void __launch_bounds__(256) dequant_rows_kernel(const int8_t* __restrict__ Wq,
                                                           const unsigned short* __restrict__ cw, int h, int o, int KT,
                                                           const int32_t* __restrict__ idx,
                                                           const int32_t* __restrict__ count, int cap,
                                                           unsigned short* __restrict__ Wo)
{
    const int j = blockIdx.x * 256 + threadIdx.x, t = blockIdx.y;
    if (j >= o) return;
    int cnt = *count;
    cnt = cnt < 0 ? 0 : (cnt > cap ? cap : cnt);
    unsigned short out = 0;
    if (t < cnt) {
        const unsigned k = (unsigned)idx[t];
        if (k < (unsigned)h) {
            const int q = Wq[((size_t)(j >> 5) * KT + (k >> 5)) * TILE_BYTES + tile_byte(j & 31, (int)(k & 31))];
            out = dequant_bits(q, cw[j]);
        }
    }
    Wo[(size_t)t * o + j] = out;
}

hipError_t launch_dequant_rows(const int8_t* Wq, const unsigned short* cw, int h, int o, const int32_t* idx,
                               const int32_t* count, int cap, unsigned short* Wo, hipStream_t st)
{
    dim3 grid((o + 255) / 256, opad_of(cap));
    dequant_rows_kernel<<<grid, 256, 0, st>>>(Wq, cw, h, o, k_tiles(h), idx, count, cap, Wo);
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
