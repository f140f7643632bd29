// Zeropoint (asymmetric) quantization, Section 2.1 Eq. 1-5, one set of constants
// per row of X and per column of W (the "zeropoint vector-wise" rows of Table 1),
// for the variant of the matmul that uses it in place of absmax quantization.
//
// For a vector with lo = min, hi = max, D = hi - lo:
//   Eq. 1  nd = 254 / D, never rounded on its own
//   Eq. 3  u(x) = round-half-even(nd x) = round-half-even(254 x / D)
//   Eq. 2  zp = u(lo) + 127 (the printed "X min" read as nd min; the 127 recentres the stored
//          byte into [-127, 127]); stored code = u(x) - zp, and Eq. 4's code + zp gives u(x) back
// D = 0 (a constant vector): codes 0, zp 0.
//
// The constants of a vector travel as one 16-byte record (ZpConst): the fp16 bit patterns of lo
// and hi, zp, and the sum of the vector's codes (the row / column sums that the unrolled product
// of Eq. 5 needs).
#include "common.h"

namespace llmint8 {

typedef unsigned short us8 __attribute__((ext_vector_type(8)));
typedef unsigned int u4 __attribute__((ext_vector_type(4)));
typedef unsigned int u2 __attribute__((ext_vector_type(2)));

// f16_key / key_f16, zp_u / zp_u_rcp and make_const live in common.h (the short-X pre-pass uses them too).

// ---------------------------------------------------------------------------
// Weights: column ranges over slabs of rows, constants, codes + column sums.
// ---------------------------------------------------------------------------
__global__ void __launch_bounds__(256) zp_colrange_partial_kernel(const unsigned short* __restrict__ W, int h, int o,
                                                                  unsigned short* __restrict__ pmin,
                                                                  unsigned short* __restrict__ pmax, int rows_per_slab)
{
    const int j = blockIdx.x * 256 + threadIdx.x;
    if (j >= o) return;
    const int r0 = blockIdx.y * rows_per_slab, r1 = min(h, r0 + rows_per_slab);
    unsigned kmin = 0xffffu, kmax = 0u;
    for (int r = r0; r < r1; r++) {
        const unsigned k = f16_key(W[(size_t)r * o + j]);
        kmin = k < kmin ? k : kmin;
        kmax = k > kmax ? k : kmax;
    }
    pmin[(size_t)blockIdx.y * o + j] = (unsigned short)kmin;
    pmax[(size_t)blockIdx.y * o + j] = (unsigned short)kmax;
}

__global__ void __launch_bounds__(256) zp_colrange_final_kernel(const unsigned short* __restrict__ pmin,
                                                                const unsigned short* __restrict__ pmax, int nslab,
                                                                int o, int4* __restrict__ zc)
{
    const int j = blockIdx.x * 256 + threadIdx.x;
    if (j >= o) return;
    unsigned kmin = 0xffffu, kmax = 0u;
    for (int sl = 0; sl < nslab; sl++) {
        const unsigned a = pmin[(size_t)sl * o + j], b = pmax[(size_t)sl * o + j];
        kmin = a < kmin ? a : kmin;
        kmax = b > kmax ? b : kmax;
    }
    zc[j] = make_const(kmin, kmax);
}

// W_i8 in the tiled layout, as quantize_weight_kernel: one workgroup = 32 features x 256 output
// columns, staged through LDS.  Also adds this slab's part of every column sum into the records.
__global__ void __launch_bounds__(256) zp_quantize_weight_kernel(const unsigned short* __restrict__ W, int h, int o,
                                                                 int4* __restrict__ zc, int8_t* __restrict__ Wq,
                                                                 int KT, int JT)
{
    __shared__ __attribute__((aligned(16))) int8_t stage[8 * TILE_BYTES];
    __shared__ int csum[256];
    const int tid = threadIdx.x;
    const int kt = blockIdx.y;
    const int jt0 = blockIdx.x * 8;
    const int cg = tid & 31, sub = tid >> 5;
    const int j0 = jt0 * 32 + cg * 8;
    csum[tid] = 0;
    double D[8], rD[8];
    int z[8], part[8];
#pragma unroll
    for (int e = 0; e < 8; e++) {
        D[e] = 0.0;
        rD[e] = 0.0;
        z[e] = 0;
        part[e] = 0;
        if (j0 + e < o) {
            const int4 r = zc[j0 + e];
            D[e] = zp_range((unsigned)r.x);
            rD[e] = D[e] > 0.0 ? 1.0 / D[e] : 0.0;
            z[e] = r.y;
        }
    }
    __syncthreads();
#pragma unroll
    for (int q = 0; q < 4; q++) {
        const int kk = q * 8 + sub;
        const int k = kt * 32 + kk;
#pragma unroll
        for (int e = 0; e < 8; e++) {
            int qv = 0;  // padding rows and columns of the tiles stay zero
            if (k < h && D[e] > 0.0) qv = zp_u_rcp(W[(size_t)k * o + j0 + e], D[e], rD[e]) - z[e];
            part[e] += qv;
            const int jj = cg * 8 + e;
            stage[(jj >> 5) * TILE_BYTES + tile_byte(jj & 31, kk)] = (int8_t)qv;
        }
    }
#pragma unroll
    for (int e = 0; e < 8; e++)
        if (part[e]) atomicAdd(&csum[cg * 8 + e], part[e]);
    __syncthreads();
    const int tile = tid >> 5;
    if (jt0 + tile < JT) {
        const u4* src = (const u4*)(stage + tid * 32);
        u4* dst = (u4*)(Wq + ((size_t)(jt0 + tile) * KT + kt) * TILE_BYTES + (tid & 31) * 32);
        dst[0] = src[0];
        dst[1] = src[1];
    }
    const int j = jt0 * 32 + tid;
    if (j < o && csum[tid]) atomicAdd(&zc[j].z, csum[tid]);
}

int zp_colrange_slabs(int h, int o)
{
    const int colblocks = (o + 255) / 256;
    int n = (2048 + colblocks - 1) / colblocks;
    const int maxslab = (h + 31) / 32;
    if (n > maxslab) n = maxslab;
    if (n > 64) n = 64;
    return n < 1 ? 1 : n;
}

hipError_t launch_zp_quantize_weight(const void* W, int h, int o, int8_t* Wq, int4* zc, unsigned short* part,
                                     hipStream_t st)
{
    const int nslab = zp_colrange_slabs(h, o);
    const int rps = (h + nslab - 1) / nslab;
    unsigned short* pmin = part;
    unsigned short* pmax = part + (size_t)nslab * o;
    zp_colrange_partial_kernel<<<dim3((o + 255) / 256, nslab), 256, 0, st>>>((const unsigned short*)W, h, o, pmin, pmax,
                                                                            rps);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    zp_colrange_final_kernel<<<(o + 255) / 256, 256, 0, st>>>(pmin, pmax, nslab, o, zc);
    e = hipGetLastError();
    if (e != hipSuccess) return e;
    const int KT = k_tiles(h), JT = row_tiles(o);
    zp_quantize_weight_kernel<<<dim3((JT + 7) / 8, KT), 256, 0, st>>>((const unsigned short*)W, h, o, zc, Wq, KT, JT);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------
// The per-column factors of Eq. 5 for column j, three planes of `pitch` doubles (see zp_kcol_kernel, which
// documents them).  idx[0 .. cnt): the outlier set, in global memory or in LDS.
// ---------------------------------------------------------------------------
__device__ __forceinline__ void zp_col_factors(const int8_t* __restrict__ Wq, const int4* __restrict__ zcw, int h, int o,
                                               int KT, const int32_t* idx, int cnt, int pitch,
                                               double* __restrict__ colc, int j)
{
    double p = 0.0, q = 0.0, r = 0.0;
    if (j < o) {
        const int4 rec = zcw[j];
        long long sum = rec.z;
        int used = 0;
        // eight codes per pass, requested without conditions so that they are in flight together (a slot past the
        // count or with an index that does not exist reads row 0 and is skipped)
        for (int t0 = 0; t0 < cnt; t0 += 8) {
            int8_t q[8];
            bool ok[8];
#pragma unroll
            for (int u = 0; u < 8; u++) {
                const unsigned k = (unsigned)idx[t0 + u < cnt ? t0 + u : 0];
                ok[u] = t0 + u < cnt && k < (unsigned)h;
                const unsigned kk = ok[u] ? k : 0u;
                q[u] = Wq[((size_t)(j >> 5) * KT + (kk >> 5)) * TILE_BYTES + tile_byte(j & 31, (int)(kk & 31))];
            }
#pragma unroll
            for (int u = 0; u < 8; u++)
                if (ok[u]) {
                    sum -= q[u];
                    used++;
                }
        }
        p = zp_range((unsigned)rec.x) * (1.0 / 254.0);
        q = (double)rec.y * p;
        r = (double)(sum + (long long)(h - used) * rec.y) * p;
    }
    colc[j] = p;
    colc[(size_t)pitch + j] = q;
    colc[2 * (size_t)pitch + j] = r;
}

// ---------------------------------------------------------------------------
// Hidden states.  One workgroup per row: range over the non-outlier columns,
// constants, and the gathered outlier columns Xo (as row_absmax_kernel).
// LISTS: the outlier set comes straight from the column lists of the scan
// (workgroup 0 then writes idx, count and status), and the workgroups past
// the s rows, cj.pitch / 256 of them, make the per-column factors of Eq. 5
// that would otherwise take a kernel of their own (cap <= JOB_MAX_CAP).
// ---------------------------------------------------------------------------
template <bool LISTS>
__global__ void __launch_bounds__(256) zp_row_range_kernel(const unsigned short* __restrict__ X, int s, int h,
                                                           int32_t* __restrict__ idx, int32_t* __restrict__ count,
                                                           int32_t* __restrict__ status, OutlierLists L, int capc,
                                                           int cap, int opad, int4* __restrict__ zc,
                                                           unsigned short* __restrict__ Xo, int vec_ok, ColumnJob cj)
{
    extern __shared__ unsigned bitmap[];  // ceil(h / 32) words, then 8 words of reduction space
    __shared__ int s_cnt[LISTS ? MAXLISTS : 1], s_base[LISTS ? MAXLISTS : 1];
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const int nw = (h + 31) / 32;
    unsigned* red = bitmap + nw;
    if constexpr (LISTS) {
        if ((int)blockIdx.x >= s) {  // a column job: the outlier set into LDS first, then one column per thread
            __shared__ int s_idx[JOB_MAX_CAP];
            const int nl = (h + 255) / 256;
            const int total = scan_lists(L.count, nl, s_cnt, s_base);
            const int cnt = total < cap ? total : cap;
            for (int b = tid; b < nl; b += 256) {
                const int n = s_cnt[b] < capc ? s_cnt[b] : capc;
                for (int e = 0; e < n && s_base[b] + e < cap; e++) s_idx[s_base[b] + e] = L.cand[(size_t)b * capc + e];
            }
            __syncthreads();
            const int j = ((int)blockIdx.x - s) * 256 + tid;
            if (j < cj.pitch)
                zp_col_factors(cj.Wq, (const int4*)cj.wconst, h, cj.o, k_tiles(h), s_idx, cnt, cj.pitch,
                               (double*)cj.out, j);
            return;
        }
    }
    const int i = blockIdx.x;
    const unsigned short* row = X + (size_t)i * h;
    for (int q = tid; q < nw; q += 256) bitmap[q] = 0;
    if constexpr (LISTS) {
        const int nl = (h + 255) / 256;
        const int total = scan_lists(L.count, nl, s_cnt, s_base);  // its barriers also publish the cleared bitmap
        const int cnt = total < cap ? total : cap;
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
        int cnt = *count;
        cnt = cnt < 0 ? 0 : (cnt > cap ? cap : cnt);
        __syncthreads();
        for (int t = tid; t < cnt; t += 256) {
            const unsigned j = (unsigned)idx[t];
            if (j < (unsigned)h) atomicOr(&bitmap[j >> 5], 1u << (j & 31));
        }
        for (int t = tid; t < opad; t += 256) {
            unsigned short v = 0;
            if (t < cnt) {
                const unsigned j = (unsigned)idx[t];
                if (j < (unsigned)h) v = row[j];
            }
            Xo[(size_t)i * opad + t] = v;
        }
    }
    __syncthreads();
    unsigned kmin = 0xffffu, kmax = 0u;
    if (vec_ok) {
        // four unconditional loads in flight per pass (past the row: its start again, skipped below)
        for (int c0 = tid * 8; c0 < h; c0 += 4 * 2048) {
            us8 v[4];
#pragma unroll
            for (int u = 0; u < 4; u++) {
                const int c = c0 + u * 2048;
                v[u] = *(const us8*)(row + (c < h ? c : 0));
            }
#pragma unroll
            for (int u = 0; u < 4; u++) {
                const int c = c0 + u * 2048;
                if (c < h) {
                    const unsigned bits = (bitmap[c >> 5] >> (c & 31)) & 0xffu;
#pragma unroll
                    for (int e = 0; e < 8; e++)
                        if (!((bits >> e) & 1u)) {
                            const unsigned k = f16_key(v[u][e]);
                            kmin = k < kmin ? k : kmin;
                            kmax = k > kmax ? k : kmax;
                        }
                }
            }
        }
    } else {
        for (int c = tid; c < h; c += 256)
            if (!((bitmap[c >> 5] >> (c & 31)) & 1u)) {
                const unsigned k = f16_key(row[c]);
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
        red[w] = kmin;
        red[4 + w] = kmax;
    }
    __syncthreads();
    if (tid == 0) {
#pragma unroll
        for (int q = 1; q < 4; q++) {
            kmin = red[q] < kmin ? red[q] : kmin;
            kmax = red[4 + q] > kmax ? red[4 + q] : kmax;
        }
        int4 r = {0, 0, 0, 0};       // no non-outlier column at all: an empty, all-zero vector
        if (kmin <= kmax) r = make_const(kmin, kmax);
        zc[i] = r;
    }
}

// X_i8 in the tiled layout, as quantize_rows_kernel, with NB = 2 blocks of 256 features per workgroup (256
// threads each): one workgroup = 32 rows x 512 features.  Also adds this workgroup's part of every row sum
// into the records, one global atomic addition per row and workgroup: these additions are what the kernel
// waits for at its end, and with half as many of them (the halves' parts meet in LDS first) it takes 17.5
// instead of 23.3 us on a 4 096 x 5 120 X, 55 us less on 2 048 x 49 152; four blocks per workgroup are no
// better (19.3 us).
constexpr int ZQ_NB = 2;

__global__ void __launch_bounds__(256 * ZQ_NB) zp_quantize_rows_kernel(const unsigned short* __restrict__ X, int s, int h,
                                                                       const int32_t* __restrict__ idx,
                                                                       const int32_t* __restrict__ count, int cap,
                                                                       int4* __restrict__ zc, int8_t* __restrict__ Xq,
                                                                       int KT, int vec_ok)
{
    constexpr int NB = ZQ_NB;
    __shared__ __attribute__((aligned(16))) int8_t stage[NB * 8 * TILE_BYTES];
    __shared__ unsigned bitmap[8 * NB];
    __shared__ int s_sum[32];
    const int tid = threadIdx.x, g = tid >> 8, t = tid & 255;
    const int rt = blockIdx.x;
    const int kw = blockIdx.y * NB * 256;  // the workgroup's first feature
    const int k0 = kw + g * 256;           // this thread's block
    if (tid < 8 * NB) bitmap[tid] = 0;
    if (tid < 32) s_sum[tid] = 0;
    int cnt = *count;
    cnt = cnt < 0 ? 0 : (cnt > cap ? cap : cnt);
    __syncthreads();
    for (int t2 = tid; t2 < cnt; t2 += 256 * NB) {
        const unsigned j = (unsigned)idx[t2] - (unsigned)kw;
        if (j < 256u * NB) atomicOr(&bitmap[j >> 5], 1u << (j & 31));
    }
    __syncthreads();
    const int kseg = (t & 31) * 8;
    const int k = k0 + kseg;
    const unsigned bits = (bitmap[g * 8 + (kseg >> 5)] >> (kseg & 31)) & 0xffu;
    // the loads of the thread's four rows first and unconditional (a row past the last one: the last one again,
    // its range taken as 0 below), so that they are in flight together, as in quantize_rows_kernel
    us8 vq[4];
    int4 recq[4];
    const bool vec = vec_ok && k + 8 <= h;
#pragma unroll
    for (int q = 0; q < 4; q++) {
        const int i = rt * 32 + q * 8 + (t >> 5);
        const int ii = i < s ? i : s - 1;
        recq[q] = zc[ii];
        vq[q] = (us8)(0);
        if (vec) vq[q] = *(const us8*)(X + (size_t)ii * h + k);
    }
#pragma unroll
    for (int q = 0; q < 4; q++) {
        const int r = q * 8 + (t >> 5);
        const int i = rt * 32 + r;
        double D = 0.0;
        int z = 0;
        us8 v = vq[q];
        if (i < s) {
            D = zp_range((unsigned)recq[q].x);
            z = recq[q].y;
            if (!vec) {
                const unsigned short* row = X + (size_t)i * h;
#pragma unroll
                for (int e = 0; e < 8; e++)
                    if (k + e < h) v[e] = row[k + e];
            }
        }
        const double rD = D > 0.0 ? 1.0 / D : 0.0;
        unsigned lo = 0, hi = 0;
        int part = 0;
#pragma unroll
        for (int e = 0; e < 8; e++) {
            int qv = 0;
            if (D > 0.0 && k + e < h && !((bits >> e) & 1u)) qv = zp_u_rcp(v[e], D, rD) - z;
            part += qv;
            const unsigned byte = (unsigned)qv & 0xffu;
            if (e < 4) lo |= byte << (8 * e); else hi |= byte << (8 * (e - 4));
        }
        u2 pk = {lo, hi};
        *(u2*)(stage + (g * 8 + (kseg >> 5)) * TILE_BYTES + tile_byte(r, kseg & 31)) = pk;
        // the 32 lanes that share row r (one half of a wave) add up their parts
#pragma unroll
        for (int d = 16; d >= 1; d >>= 1) part += __shfl_xor(part, d);
        if ((t & 31) == 0 && i < s && part) atomicAdd(&s_sum[r], part);
    }
    __syncthreads();
    if (tid < 32 && rt * 32 + tid < s && s_sum[tid]) atomicAdd(&zc[rt * 32 + tid].z, s_sum[tid]);
    const int kt0 = kw >> 5;
#pragma unroll
    for (int half = 0; half < 2; half++) {
        const int off = half * (NB * 4096) + tid * 16;
        if (kt0 + (off >> 10) < KT)
            *(u4*)(Xq + ((size_t)rt * KT + kt0) * TILE_BYTES + off) = *(const u4*)(stage + off);
    }
}

static hipError_t launch_zp_codes(const void* X, int s, int h, const int32_t* idx, const int32_t* count, int cap,
                                  int8_t* Xq, int4* zc, int vec_ok, hipStream_t st)
{
    const int KT = k_tiles(h), RT = row_tiles(s);
    const int nblocks = (KT * 32 + 255) / 256;
    zp_quantize_rows_kernel<<<dim3(RT, (nblocks + ZQ_NB - 1) / ZQ_NB), 256 * ZQ_NB, 0, st>>>(
        (const unsigned short*)X, s, h, idx, count, cap, zc, Xq, KT, vec_ok);
    return hipGetLastError();
}

hipError_t launch_zp_quantize_rows(const void* X, int s, int h, const int32_t* idx, const int32_t* count, int cap,
                                   int8_t* Xq, int4* zc, unsigned short* Xo, hipStream_t st)
{
    const size_t shm = ((size_t)(h + 31) / 32 + 8) * sizeof(unsigned);
    const int vec_ok = (h % 8 == 0) && (((uintptr_t)X & 15) == 0);
    const OutlierLists none = {nullptr, nullptr, nullptr};
    const ColumnJob nojob = {nullptr, nullptr, nullptr, 0, 0};
    zp_row_range_kernel<false><<<s, 256, shm, st>>>((const unsigned short*)X, s, h, (int32_t*)idx, (int32_t*)count,
                                                    nullptr, none, 0, cap, opad_of(cap), zc, Xo, vec_ok, nojob);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    return launch_zp_codes(X, s, h, idx, count, cap, Xq, zc, vec_ok, st);
}

// the same fed by the column lists of the scan: also writes idx, count, status, and (cj, cap <= JOB_MAX_CAP)
// the per-column factors of launch_zp_kcol
hipError_t launch_zp_quantize_rows_lists(const void* X, int s, int h, OutlierLists L, int32_t* idx, int32_t* count,
                                         int32_t* status, int cap, int8_t* Xq, int4* zc, unsigned short* Xo,
                                         const ColumnJob* cj, hipStream_t st)
{
    const size_t shm = ((size_t)(h + 31) / 32 + 8) * sizeof(unsigned);
    const int vec_ok = (h % 8 == 0) && (((uintptr_t)X & 15) == 0);
    const ColumnJob job = (cj && cap <= JOB_MAX_CAP) ? *cj : ColumnJob{nullptr, nullptr, nullptr, 0, 0};
    zp_row_range_kernel<true><<<s + job.pitch / 256, 256, shm, st>>>((const unsigned short*)X, s, h, idx, count, status,
                                                                     L, list_capacity(cap), cap, opad_of(cap), zc, Xo,
                                                                     vec_ok, job);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    return launch_zp_codes(X, s, h, idx, count, cap, Xq, zc, vec_ok, st);
}

// ---------------------------------------------------------------------------
// Per call, per output column, what the GEMM epilogues multiply with (three planes of `pitch` doubles,
// zero for j >= o so that the epilogues need no guards):
//   plane 0  p[j] = D_w[j] / 254                       (1 / nd_w)
//   plane 1  q[j] = zp_w[j] * p[j]
//   plane 2  r[j] = K[j] * p[j],  K[j] = sum_{k not in O} W_i8[k][j] + (h - |O|) zp_w[j]
// so that T / nd_w of Eq. 5 is  C p + rowsum q + zp_x r.
// ---------------------------------------------------------------------------
__global__ void __launch_bounds__(256) zp_kcol_kernel(const int8_t* __restrict__ Wq, const int4* __restrict__ zcw, int h,
                                                      int o, int KT, const int32_t* __restrict__ idx,
                                                      const int32_t* __restrict__ count, int cap, int pitch,
                                                      double* __restrict__ colc)
{
    const int j = blockIdx.x * 256 + threadIdx.x;
    if (j >= pitch) return;
    int cnt = *count;
    cnt = cnt < 0 ? 0 : (cnt > cap ? cap : cnt);
    zp_col_factors(Wq, zcw, h, o, KT, idx, cnt, pitch, colc, j);
}

hipError_t launch_zp_kcol(const int8_t* Wq, const int4* zcw, int h, int o, const int32_t* idx, const int32_t* count,
                          int cap, double* colc, hipStream_t st)
{
    const int pitch = zp_col_pitch(o);
    zp_kcol_kernel<<<pitch / 256, 256, 0, st>>>(Wq, zcw, h, o, k_tiles(h), idx, count, cap, pitch, colc);
    return hipGetLastError();
}

}  // namespace llmint8
