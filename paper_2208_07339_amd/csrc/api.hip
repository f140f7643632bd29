// C-ABI entry points of libllmint8: argument checks, workspace carving and the
// kernel sequences.  Declarations and argument contracts: include/llmint8.h.
#include <atomic>
#include <cmath>
#include <mutex>

#include "../../include/llmint8.h"
#include "common.h"

using namespace llmint8;

namespace {

inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }
inline bool misaligned(const void* p, size_t a) { return ((uintptr_t)p & (a - 1)) != 0; }
inline void* ws_base(void* ws) { return (void*)align_up((uintptr_t)ws, 256); }

// outlier scan: list scratch first, then the slab maxima
inline size_t scratch_ws(int h, int cap) { return align_up(outlier_lists_bytes(h, cap), 256); }
inline size_t slab_ws(int s, int h) { return align_up((size_t)colmax_slabs(s, h) * h * 2, 256); }
// partial row maxima of the fused column / row scan: [ceil(h / 512)][s] fp16 bits
inline size_t rowpart_ws(int s, int h) { return align_up((size_t)((h + 511) / 512) * s * 2, 256); }
inline size_t outlier_ws(int s, int h, int cap) { return scratch_ws(h, cap) + slab_ws(s, h) + rowpart_ws(s, h); }
inline size_t weight_ws(int h, int o) { return align_up((size_t)colmax_slabs(h, o) * o * 2, 256); }
// rebuilt outlier rows of W (used when no fp16 weights are given): [opad x o] fp16, behind everything else
inline size_t rows_ws(int o, int cap) { return align_up((size_t)opad_of(cap) * o * 2, 256); }
// zeropoint variant: column minima and maxima of the weight scan; per call the column factors K [o] doubles
inline size_t zp_weight_ws(int h, int o) { return align_up((size_t)2 * zp_colrange_slabs(h, o) * o * 2, 256); }
inline size_t kcol_ws(int o) { return (size_t)3 * zp_col_pitch(o) * 8; }
inline size_t scan_ws(int s, int h, int o, int cap)
{
    const size_t a = outlier_ws(s, h, cap), b = weight_ws(h, o), c = zp_weight_ws(h, o);
    const size_t m = a > b ? a : b;
    return m > c ? m : c;
}

thread_local hipError_t g_last_hip = hipSuccess;  // reported by llmint8_last_hip_error()

inline int hip_status(hipError_t e)
{
    if (e == hipSuccess) return LLMINT8_OK;
    g_last_hip = e;
    return LLMINT8_HIP;
}

}  // namespace

// Scratch of llmint8_linear_static: one array per device that loads this library, held until the process
// ends.  In host code the array's name is only a handle for hipGetSymbolAddress; the address it yields
// (per device, looked up once with that device current) is what kernels and host calls are given.
static __device__ __align__(256) unsigned char scratch[LLMINT8_STATIC_SCRATCH_BYTES];

namespace {

constexpr int SCRATCH_DEVICES = 64;
std::atomic<void*> g_scratch_ptr[SCRATCH_DEVICES];
std::mutex g_scratch_lock;

// device address of `scratch` on the current device
hipError_t static_scratch(void** out)
{
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= SCRATCH_DEVICES) return hipErrorInvalidDevice;
    void* p = g_scratch_ptr[dev].load(std::memory_order_acquire);
    if (!p) {
        std::lock_guard<std::mutex> hold(g_scratch_lock);
        p = g_scratch_ptr[dev].load(std::memory_order_acquire);
        if (!p) {
            e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
            if (e != hipSuccess) return e;
            if (!p) return hipErrorInvalidSymbol;
            g_scratch_ptr[dev].store(p, std::memory_order_release);
        }
    }
    *out = p;
    return hipSuccess;
}

}  // namespace

extern "C" {

const char* llmint8_status_string(int status)
{
    switch (status) {
        case LLMINT8_OK: return "ok";
        case LLMINT8_INVALID_ARG: return "invalid argument (null or misaligned pointer, non-positive size)";
        case LLMINT8_SHAPE: return "unsupported shape (feature dimension above the int32 accumulation bound)";
        case LLMINT8_WORKSPACE: return "workspace too small";
        case LLMINT8_HIP: return "HIP launch error";
        case LLMINT8_STATIC_LIMIT:
            return "sizes need more scratch than the library's static buffer holds (use the entry point that "
                   "takes a caller's workspace)";
        default: return "unknown status";
    }
}

const char* llmint8_last_hip_error(void) { return hipGetErrorString(g_last_hip); }

int llmint8_opad(int cap) { return cap < 1 ? 0 : opad_of(cap); }

size_t llmint8_wq_bytes(int h, int o)
{
    if (h < 1 || o < 1) return 0;
    return (size_t)row_tiles(o) * k_tiles(h) * TILE_BYTES;
}

size_t llmint8_xq_bytes(int s, int h)
{
    if (s < 1 || h < 1) return 0;
    return (size_t)row_tiles(s) * k_tiles(h) * TILE_BYTES;
}

size_t llmint8_workspace_bytes(int s, int h, int o, int cap)
{
    if (s < 1 || h < 1 || o < 1 || cap < 1) return 0;
    return scan_ws(s, h, o, cap) + rows_ws(o, cap) + kcol_ws(o) + 256;  // slack to align the caller's pointer
}

static inline bool bad_granularity(int g) { return g < LLMINT8_VECTORWISE || g > LLMINT8_TENSORWISE; }

int llmint8_quantize_weight_granular(const void* W_f16, int h, int o, int granularity, int8_t* Wq, void* cw_f16,
                                     void* ws, size_t ws_bytes, llmint8_stream_t stream)
{
    if (!W_f16 || !Wq || !cw_f16 || !ws || h < 1 || o < 1 || bad_granularity(granularity))
        return LLMINT8_INVALID_ARG;
    if (misaligned(W_f16, 2) || misaligned(Wq, 16) || misaligned(cw_f16, 8)) return LLMINT8_INVALID_ARG;
    if (h > LLMINT8_MAX_H) return LLMINT8_SHAPE;
    if (ws_bytes < weight_ws(h, o) + 256) return LLMINT8_WORKSPACE;
    hipStream_t st = (hipStream_t)stream;
    unsigned short* part = (unsigned short*)ws_base(ws);
    const int nslab = colmax_slabs(h, o);
    hipError_t e = launch_colmax_partial(W_f16, h, o, part, nslab, st);
    if (e == hipSuccess) e = launch_colmax_final(part, nslab, o, (unsigned short*)cw_f16, st);
    if (e == hipSuccess && granularity != LLMINT8_VECTORWISE) e = launch_spread_max((unsigned short*)cw_f16, o, st);
    if (e == hipSuccess) e = launch_quantize_weight(W_f16, h, o, (const unsigned short*)cw_f16, Wq, st);
    return hip_status(e);
}

int llmint8_quantize_weight(const void* W_f16, int h, int o, int8_t* Wq, void* cw_f16, void* ws, size_t ws_bytes,
                            llmint8_stream_t stream)
{
    return llmint8_quantize_weight_granular(W_f16, h, o, LLMINT8_VECTORWISE, Wq, cw_f16, ws, ws_bytes, stream);
}

int llmint8_find_outliers(const void* X_f16, int s, int h, float alpha, int32_t* idx, int cap, int32_t* count,
                          int32_t* status, void* ws, size_t ws_bytes, llmint8_stream_t stream)
{
    if (!X_f16 || !idx || !count || !ws || s < 1 || h < 1 || cap < 1) return LLMINT8_INVALID_ARG;
    if (misaligned(X_f16, 2) || misaligned(idx, 4) || misaligned(count, 4) || misaligned(status, 4))
        return LLMINT8_INVALID_ARG;
    if (h > LLMINT8_MAX_H) return LLMINT8_SHAPE;
    if (ws_bytes < outlier_ws(s, h, cap) + 256) return LLMINT8_WORKSPACE;
    hipStream_t st = (hipStream_t)stream;
    char* base = (char*)ws_base(ws);
    const OutlierLists L = carve_outlier_lists(base, h, cap);
    unsigned short* part = (unsigned short*)(base + scratch_ws(h, cap));
    const int nslab = colmax_slabs(s, h);
    hipError_t e = launch_colmax_partial(X_f16, s, h, part, nslab, st);
    if (e == hipSuccess) e = launch_outlier_lists(part, nslab, h, threshold_bits(alpha), L, cap, st);
    if (e == hipSuccess) e = launch_merge_lists(L, h, idx, cap, count, status, st);
    return hip_status(e);
}

int llmint8_quantize_rows_granular(const void* X_f16, int s, int h, const int32_t* idx, const int32_t* count, int cap,
                                   int granularity, int8_t* Xq, void* cx_f16, void* Xo_f16, llmint8_stream_t stream)
{
    if (!X_f16 || !idx || !count || !Xq || !cx_f16 || !Xo_f16 || s < 1 || h < 1 || cap < 1 ||
        bad_granularity(granularity))
        return LLMINT8_INVALID_ARG;
    if (misaligned(X_f16, 2) || misaligned(idx, 4) || misaligned(count, 4) || misaligned(Xq, 16) ||
        misaligned(cx_f16, 2) || misaligned(Xo_f16, 16))
        return LLMINT8_INVALID_ARG;
    if (h > LLMINT8_MAX_H) return LLMINT8_SHAPE;
    return hip_status(launch_quantize_rows(X_f16, s, h, idx, count, cap, Xq, (unsigned short*)cx_f16,
                                           (unsigned short*)Xo_f16, granularity == LLMINT8_TENSORWISE,
                                           (hipStream_t)stream));
}

int llmint8_quantize_rows(const void* X_f16, int s, int h, const int32_t* idx, const int32_t* count, int cap,
                          int8_t* Xq, void* cx_f16, void* Xo_f16, llmint8_stream_t stream)
{
    return llmint8_quantize_rows_granular(X_f16, s, h, idx, count, cap, LLMINT8_VECTORWISE, Xq, cx_f16, Xo_f16,
                                          stream);
}

int llmint8_dequantize_rows(const int8_t* Wq, const void* cw_f16, int h, int o, const int32_t* idx,
                            const int32_t* count, int cap, void* Wo_f16, llmint8_stream_t stream)
{
    if (!Wq || !cw_f16 || !idx || !count || !Wo_f16 || h < 1 || o < 1 || cap < 1) return LLMINT8_INVALID_ARG;
    if (misaligned(Wq, 16) || misaligned(cw_f16, 2) || misaligned(idx, 4) || misaligned(count, 4) ||
        misaligned(Wo_f16, 16))
        return LLMINT8_INVALID_ARG;
    if (h > LLMINT8_MAX_H) return LLMINT8_SHAPE;
    return hip_status(launch_dequant_rows(Wq, (const unsigned short*)cw_f16, h, o, idx, count, cap,
                                          (unsigned short*)Wo_f16, (hipStream_t)stream));
}

// have_rows: with no 16-bit weights, the rebuilt outlier rows are in the workspace already (the short-X
// pre-pass of llmint8_linear makes them)
static int matmul_impl(const int8_t* Xq, const void* cx_f16, const void* Xo_f16, const int32_t* idx,
                       const int32_t* count, int cap, const int8_t* Wq, const void* cw_f16, const void* W_f16, int s,
                       int h, int o, void* Out_f16, int32_t* C_i32_debug, void* ws, size_t ws_bytes,
                       llmint8_stream_t stream, bool have_rows)
{
    if (!Xq || !cx_f16 || !Xo_f16 || !idx || !count || !Wq || !cw_f16 || !Out_f16 || s < 1 || h < 1 || o < 1 ||
        cap < 1)
        return LLMINT8_INVALID_ARG;
    if (misaligned(Xq, 16) || misaligned(Wq, 16) || misaligned(Xo_f16, 16) || misaligned(cw_f16, 8) ||
        misaligned(cx_f16, 2) || misaligned(W_f16, 2) || misaligned(Out_f16, 8) || misaligned(idx, 4) ||
        misaligned(count, 4) || misaligned(C_i32_debug, 4))
        return LLMINT8_INVALID_ARG;
    if (h > LLMINT8_MAX_H) return LLMINT8_SHAPE;
    hipStream_t st = (hipStream_t)stream;
    hipError_t e = hipSuccess;
    const unsigned short* Wrows = (const unsigned short*)W_f16;
    int rows_are_slots = 0;
    if (!W_f16) {
        // no 16-bit weights kept: rebuild the outlier rows from the codes into the workspace
        if (!ws) return LLMINT8_INVALID_ARG;
        if (ws_bytes < llmint8_workspace_bytes(s, h, o, cap)) return LLMINT8_WORKSPACE;
        unsigned short* Wo = (unsigned short*)((char*)ws_base(ws) + scan_ws(s, h, o, cap));
        if (!have_rows) e = launch_dequant_rows(Wq, (const unsigned short*)cw_f16, h, o, idx, count, cap, Wo, st);
        if (e != hipSuccess) return hip_status(e);
        Wrows = Wo;
        rows_are_slots = 1;
    }
    if (decode_kernel_takes(s, h, o, false))
        e = launch_gemm_decode(Xq, (const unsigned short*)cx_f16, (const unsigned short*)Xo_f16, count, cap, Wq,
                               (const unsigned short*)cw_f16, Wrows, rows_are_slots, idx, s, h, o,
                               (unsigned short*)Out_f16, C_i32_debug, st);
    else
        e = launch_gemm_prefill(Xq, (const unsigned short*)cx_f16, (const unsigned short*)Xo_f16, count, cap, Wq,
                                (const unsigned short*)cw_f16, Wrows, rows_are_slots, idx, s, h, o,
                                (unsigned short*)Out_f16, C_i32_debug, st);
    return hip_status(e);
}

int llmint8_matmul(const int8_t* Xq, const void* cx_f16, const void* Xo_f16, const int32_t* idx,
                   const int32_t* count, int cap, const int8_t* Wq, const void* cw_f16, const void* W_f16, int s,
                   int h, int o, void* Out_f16, int32_t* C_i32_debug, void* ws, size_t ws_bytes,
                   llmint8_stream_t stream)
{
    return matmul_impl(Xq, cx_f16, Xo_f16, idx, count, cap, Wq, cw_f16, W_f16, s, h, o, Out_f16, C_i32_debug, ws,
                       ws_bytes, stream, false);
}

static int linear_impl(const void* X_f16, int s, int h, float alpha, int granularity, const int8_t* Wq, const void* cw_f16,
                       const void* W_f16, int o, int32_t* idx, int cap, int32_t* count, int32_t* status, int8_t* Xq,
                       void* cx_f16, void* Xo_f16, void* Out_f16, void* ws, size_t ws_bytes, llmint8_stream_t stream,
                       hipEvent_t ev_before, hipEvent_t ev_after)
{
    // validate everything before anything is enqueued
    if (!X_f16 || !idx || !count || !ws || !Xq || !cx_f16 || !Xo_f16 || !Wq || !cw_f16 || !Out_f16 || s < 1 || h < 1 ||
        o < 1 || cap < 1 || bad_granularity(granularity))
        return LLMINT8_INVALID_ARG;
    if (misaligned(X_f16, 2) || misaligned(idx, 4) || misaligned(count, 4) || misaligned(status, 4) ||
        misaligned(Xq, 16) || misaligned(Wq, 16) || misaligned(Xo_f16, 16) || misaligned(cw_f16, 8) ||
        misaligned(cx_f16, 2) || misaligned(W_f16, 2) || misaligned(Out_f16, 8))
        return LLMINT8_INVALID_ARG;
    if (h > LLMINT8_MAX_H) return LLMINT8_SHAPE;
    if (ws_bytes < llmint8_workspace_bytes(s, h, o, cap)) return LLMINT8_WORKSPACE;
    // Same results as llmint8_find_outliers + llmint8_quantize_rows, in fewer kernels: the row
    // constants and the quantizer read the column lists of the scan directly.
    hipStream_t st = (hipStream_t)stream;
    char* base = (char*)ws_base(ws);
    const OutlierLists L = carve_outlier_lists(base, h, cap);
    // the constants of W were fixed when it was quantized; here only those of X depend on the granularity
    const int shared_cx = granularity == LLMINT8_TENSORWISE;
    hipError_t e;
    if (s <= 32) {
        // without 16-bit weights the second kernel also rebuilds the outlier rows of W from the codes
        const ColumnJob job = {Wq, cw_f16, base + scan_ws(s, h, o, cap), o, (o + 255) & ~255};
        e = launch_prepass_small(X_f16, s, h, threshold_bits(alpha), L, idx, cap, count, status,
                                 (unsigned short*)cx_f16, (unsigned short*)Xo_f16, Xq, shared_cx, st, nullptr,
                                 W_f16 ? nullptr : &job);
    } else {
        if (std::isinf(alpha) && alpha > 0.0f) {
            // no decomposition (the baselines of Table 1 without it): O is empty, X need not be scanned
            e = launch_clear_lists(L, h, st);
            if (e == hipSuccess)
                e = launch_quantize_rows_lists(X_f16, s, h, L, idx, count, status, cap, Xq, (unsigned short*)cx_f16,
                                               (unsigned short*)Xo_f16, shared_cx, st);
        } else {
            unsigned short* part = (unsigned short*)(base + scratch_ws(h, cap));
            const int nslab = colmax_slabs(s, h);
            const unsigned thr = threshold_bits(alpha);
            if (!shared_cx && h % 8 == 0 && !misaligned(X_f16, 16)) {
                // X is read twice instead of three times: the column scan leaves partial row maxima, from which
                // a small kernel gets the row constants once the outlier columns are known
                unsigned short* rowpart = (unsigned short*)(base + scratch_ws(h, cap) + slab_ws(s, h));
                e = launch_colmax_rowmax(X_f16, s, h, part, nslab, rowpart, thr, st);
                if (e == hipSuccess) e = launch_outlier_lists(part, nslab, h, thr, L, cap, st);
                if (e == hipSuccess)
                    e = launch_quantize_rows_rowpart(X_f16, s, h, L, thr, rowpart, idx, count, status, cap, Xq,
                                                     (unsigned short*)cx_f16, (unsigned short*)Xo_f16, st);
            } else {
                e = launch_colmax_partial(X_f16, s, h, part, nslab, st);
                if (e == hipSuccess) e = launch_outlier_lists(part, nslab, h, thr, L, cap, st);
                if (e == hipSuccess)
                    e = launch_quantize_rows_lists(X_f16, s, h, L, idx, count, status, cap, Xq,
                                                   (unsigned short*)cx_f16, (unsigned short*)Xo_f16, shared_cx, st);
            }
        }
    }
    if (e == hipSuccess && ev_before) e = hipEventRecord(ev_before, st);
    if (e != hipSuccess) return hip_status(e);
    const int r = matmul_impl(Xq, cx_f16, Xo_f16, idx, count, cap, Wq, cw_f16, W_f16, s, h, o, Out_f16, nullptr, ws,
                              ws_bytes, stream, s <= 32 && cap <= JOB_MAX_CAP);
    if (r == LLMINT8_OK && ev_after) return hip_status(hipEventRecord(ev_after, st));
    return r;
}

int llmint8_linear(const void* X_f16, int s, int h, float alpha, const int8_t* Wq, const void* cw_f16,
                   const void* W_f16, int o, int32_t* idx, int cap, int32_t* count, int32_t* status, int8_t* Xq,
                   void* cx_f16, void* Xo_f16, void* Out_f16, void* ws, size_t ws_bytes, llmint8_stream_t stream)
{
    return linear_impl(X_f16, s, h, alpha, LLMINT8_VECTORWISE, Wq, cw_f16, W_f16, o, idx, cap, count, status, Xq,
                       cx_f16, Xo_f16, Out_f16, ws, ws_bytes, stream, nullptr, nullptr);
}

int llmint8_linear_granular(const void* X_f16, int s, int h, float alpha, int granularity, const int8_t* Wq,
                            const void* cw_f16, const void* W_f16, int o, int32_t* idx, int cap, int32_t* count,
                            int32_t* status, int8_t* Xq, void* cx_f16, void* Xo_f16, void* Out_f16, void* ws,
                            size_t ws_bytes, llmint8_stream_t stream)
{
    return linear_impl(X_f16, s, h, alpha, granularity, Wq, cw_f16, W_f16, o, idx, cap, count, status, Xq, cx_f16,
                       Xo_f16, Out_f16, ws, ws_bytes, stream, nullptr, nullptr);
}

int llmint8_linear_events(const void* X_f16, int s, int h, float alpha, int granularity, const int8_t* Wq, const void* cw_f16,
                          const void* W_f16, int o, int32_t* idx, int cap, int32_t* count, int32_t* status,
                          int8_t* Xq, void* cx_f16, void* Xo_f16, void* Out_f16, void* ws, size_t ws_bytes,
                          llmint8_stream_t stream, void* ev_before_matmul, void* ev_after_matmul)
{
    return linear_impl(X_f16, s, h, alpha, granularity, Wq, cw_f16, W_f16, o, idx, cap, count, status, Xq, cx_f16,
                       Xo_f16, Out_f16, ws, ws_bytes, stream, (hipEvent_t)ev_before_matmul,
                       (hipEvent_t)ev_after_matmul);
}

// ---- one-time set-up, and the entry point that allocates nothing --------------

int llmint8_init(void)
{
    int cus = 0;
    hipError_t e = prefill_device_setup(&cus);
    if (e != hipSuccess) return hip_status(e);
    void* p = nullptr;
    return hip_status(static_scratch(&p));
}

int llmint8_linear_static(const void* X_f16, int s, int h, float alpha, const int8_t* Wq, const void* cw_f16,
                          const void* W_f16, int o, int32_t* idx, int cap, int32_t* count, int32_t* status, int8_t* Xq,
                          void* cx_f16, void* Xo_f16, void* Out_f16, llmint8_stream_t stream)
{
    if (s < 1 || h < 1 || o < 1 || cap < 1) return LLMINT8_INVALID_ARG;
    if (h > LLMINT8_MAX_H) return LLMINT8_SHAPE;
    if (llmint8_workspace_bytes(s, h, o, cap) > (size_t)LLMINT8_STATIC_SCRATCH_BYTES) return LLMINT8_STATIC_LIMIT;
    void* p = nullptr;
    const hipError_t e = static_scratch(&p);
    if (e != hipSuccess) return hip_status(e);
    // Nothing in the scratch has to start at zero: every kernel of the sequence reads only what a kernel
    // earlier in the same call wrote (list counts and entries, slab maxima, partial row maxima, rebuilt rows).
    return linear_impl(X_f16, s, h, alpha, LLMINT8_VECTORWISE, Wq, cw_f16, W_f16, o, idx, cap, count, status, Xq,
                       cx_f16, Xo_f16, Out_f16, p, (size_t)LLMINT8_STATIC_SCRATCH_BYTES, stream, nullptr, nullptr);
}

// ---- zeropoint variant ------------------------------------------------------

int llmint8_zp_quantize_weight(const void* W_f16, int h, int o, int8_t* Wq, int32_t* zc_w, void* ws, size_t ws_bytes,
                               llmint8_stream_t stream)
{
    if (!W_f16 || !Wq || !zc_w || !ws || h < 1 || o < 1) return LLMINT8_INVALID_ARG;
    if (misaligned(W_f16, 2) || misaligned(Wq, 16) || misaligned(zc_w, 16)) return LLMINT8_INVALID_ARG;
    if (h > LLMINT8_MAX_H) return LLMINT8_SHAPE;
    if (ws_bytes < zp_weight_ws(h, o) + 256) return LLMINT8_WORKSPACE;
    return hip_status(launch_zp_quantize_weight(W_f16, h, o, Wq, (int4*)zc_w, (unsigned short*)ws_base(ws),
                                                (hipStream_t)stream));
}

int llmint8_zp_quantize_rows(const void* X_f16, int s, int h, const int32_t* idx, const int32_t* count, int cap,
                             int8_t* Xq, int32_t* zc_x, void* Xo_f16, llmint8_stream_t stream)
{
    if (!X_f16 || !idx || !count || !Xq || !zc_x || !Xo_f16 || s < 1 || h < 1 || cap < 1) return LLMINT8_INVALID_ARG;
    if (misaligned(X_f16, 2) || misaligned(idx, 4) || misaligned(count, 4) || misaligned(Xq, 16) ||
        misaligned(zc_x, 16) || misaligned(Xo_f16, 16))
        return LLMINT8_INVALID_ARG;
    if (h > LLMINT8_MAX_H) return LLMINT8_SHAPE;
    return hip_status(launch_zp_quantize_rows(X_f16, s, h, idx, count, cap, Xq, (int4*)zc_x, (unsigned short*)Xo_f16,
                                              (hipStream_t)stream));
}

// have_factors: the per-column factors of Eq. 5 are in the workspace already (the short-X pre-pass of
// llmint8_zp_linear makes them)
static int zp_matmul_impl(const int8_t* Xq, const int32_t* zc_x, const void* Xo_f16, const int32_t* idx,
                          const int32_t* count, int cap, const int8_t* Wq, const int32_t* zc_w, const void* W_f16, int s,
                          int h, int o, void* Out_f16, int32_t* C_i32_debug, void* ws, size_t ws_bytes,
                          llmint8_stream_t stream, bool have_factors)
{
    if (!Xq || !zc_x || !Xo_f16 || !idx || !count || !Wq || !zc_w || !W_f16 || !Out_f16 || !ws || s < 1 || h < 1 ||
        o < 1 || cap < 1)
        return LLMINT8_INVALID_ARG;
    if (misaligned(Xq, 16) || misaligned(Wq, 16) || misaligned(Xo_f16, 16) || misaligned(zc_x, 16) ||
        misaligned(zc_w, 16) || misaligned(W_f16, 2) || misaligned(Out_f16, 8) || misaligned(idx, 4) ||
        misaligned(count, 4) || misaligned(C_i32_debug, 4))
        return LLMINT8_INVALID_ARG;
    if (h > LLMINT8_MAX_H) return LLMINT8_SHAPE;
    if (ws_bytes < llmint8_workspace_bytes(s, h, o, cap)) return LLMINT8_WORKSPACE;
    hipStream_t st = (hipStream_t)stream;
    double* kcol = (double*)((char*)ws_base(ws) + scan_ws(s, h, o, cap) + rows_ws(o, cap));
    hipError_t e = hipSuccess;
    if (!have_factors) e = launch_zp_kcol(Wq, (const int4*)zc_w, h, o, idx, count, cap, kcol, st);
    if (e != hipSuccess) return hip_status(e);
    const ZpArgs zp = {(const int4*)zc_x, kcol, zp_col_pitch(o)};
    if (decode_kernel_takes(s, h, o, true))
        e = launch_gemm_decode(Xq, nullptr, (const unsigned short*)Xo_f16, count, cap, Wq, nullptr,
                               (const unsigned short*)W_f16, 0, idx, s, h, o, (unsigned short*)Out_f16, C_i32_debug,
                               st, &zp);
    else
        e = launch_gemm_prefill(Xq, nullptr, (const unsigned short*)Xo_f16, count, cap, Wq, nullptr,
                                (const unsigned short*)W_f16, 0, idx, s, h, o, (unsigned short*)Out_f16, C_i32_debug,
                                st, &zp);
    return hip_status(e);
}

int llmint8_zp_matmul(const int8_t* Xq, const int32_t* zc_x, const void* Xo_f16, const int32_t* idx,
                      const int32_t* count, int cap, const int8_t* Wq, const int32_t* zc_w, const void* W_f16, int s,
                      int h, int o, void* Out_f16, int32_t* C_i32_debug, void* ws, size_t ws_bytes,
                      llmint8_stream_t stream)
{
    return zp_matmul_impl(Xq, zc_x, Xo_f16, idx, count, cap, Wq, zc_w, W_f16, s, h, o, Out_f16, C_i32_debug, ws,
                          ws_bytes, stream, false);
}

int llmint8_zp_linear(const void* X_f16, int s, int h, float alpha, const int8_t* Wq, const int32_t* zc_w,
                      const void* W_f16, int o, int32_t* idx, int cap, int32_t* count, int32_t* status, int8_t* Xq,
                      int32_t* zc_x, void* Xo_f16, void* Out_f16, void* ws, size_t ws_bytes, llmint8_stream_t stream)
{
    if (!X_f16 || !idx || !count || !ws || !Xq || !zc_x || !Xo_f16 || !Wq || !zc_w || !W_f16 || !Out_f16 || s < 1 ||
        h < 1 || o < 1 || cap < 1)
        return LLMINT8_INVALID_ARG;
    if (misaligned(X_f16, 2) || misaligned(idx, 4) || misaligned(count, 4) || misaligned(status, 4) ||
        misaligned(Xq, 16) || misaligned(Wq, 16) || misaligned(Xo_f16, 16) || misaligned(zc_x, 16) ||
        misaligned(zc_w, 16) || misaligned(W_f16, 2) || misaligned(Out_f16, 8))
        return LLMINT8_INVALID_ARG;
    if (h > LLMINT8_MAX_H) return LLMINT8_SHAPE;
    if (ws_bytes < llmint8_workspace_bytes(s, h, o, cap)) return LLMINT8_WORKSPACE;
    int r;
    if (s <= 32) {
        // short X: outlier scan, records, codes and gathered columns in two kernels (the same results as the
        // two calls below); the second one also makes the per-column factors the matmul kernel needs
        const OutlierLists L = carve_outlier_lists((char*)ws_base(ws), h, cap);
        const ColumnJob job = {Wq, zc_w, (char*)ws_base(ws) + scan_ws(s, h, o, cap) + rows_ws(o, cap), o,
                               zp_col_pitch(o)};
        r = hip_status(launch_prepass_small(X_f16, s, h, threshold_bits(alpha), L, idx, cap, count, status, nullptr,
                                            (unsigned short*)Xo_f16, Xq, 0, (hipStream_t)stream, (int4*)zc_x, &job));
    } else {
        // the column scan as llmint8_find_outliers runs it, without its last kernel: the kernel that takes the
        // rows' ranges reads the column lists itself, writes idx / count / status, and carries the per-column
        // factors of the matmul as extra workgroups
        hipStream_t st = (hipStream_t)stream;
        char* base = (char*)ws_base(ws);
        const OutlierLists L = carve_outlier_lists(base, h, cap);
        unsigned short* part = (unsigned short*)(base + scratch_ws(h, cap));
        const int nslab = colmax_slabs(s, h);
        const ColumnJob job = {Wq, zc_w, base + scan_ws(s, h, o, cap) + rows_ws(o, cap), o, zp_col_pitch(o)};
        hipError_t e = launch_colmax_partial(X_f16, s, h, part, nslab, st);
        if (e == hipSuccess) e = launch_outlier_lists(part, nslab, h, threshold_bits(alpha), L, cap, st);
        if (e == hipSuccess)
            e = launch_zp_quantize_rows_lists(X_f16, s, h, L, idx, count, status, cap, Xq, (int4*)zc_x,
                                              (unsigned short*)Xo_f16, &job, st);
        r = hip_status(e);
    }
    if (r == LLMINT8_OK)
        r = zp_matmul_impl(Xq, zc_x, Xo_f16, idx, count, cap, Wq, zc_w, W_f16, s, h, o, Out_f16, nullptr, ws, ws_bytes,
                           stream, cap <= JOB_MAX_CAP);
    return r;
}

int llmint8_debug_prefill_tile(int cfg)
{
    if (cfg < -1 || cfg >= LLMINT8_PREFILL_TILES) return LLMINT8_INVALID_ARG;
    g_force_cfg.store(cfg, std::memory_order_relaxed);
    return LLMINT8_OK;
}

int llmint8_debug_prefill_tile_for(int s, int h, int o)
{
    if (s < 1 || h < 1 || o < 1) return -1;
    return pick_cfg(s, h, o);
}

int llmint8_debug_decode_shape(int cfg)
{
    if (cfg < -1 || cfg > LLMINT8_DECODE_SHAPES) return LLMINT8_INVALID_ARG;
    g_decode_cfg.store(cfg, std::memory_order_relaxed);
    return LLMINT8_OK;
}

int llmint8_export_weight(const int8_t* Wq, int h, int o, int8_t* W_i8_rowmajor, llmint8_stream_t stream)
{
    if (!Wq || !W_i8_rowmajor || h < 1 || o < 1 || misaligned(Wq, 16)) return LLMINT8_INVALID_ARG;
    return hip_status(launch_export_tiled(Wq, o, h, W_i8_rowmajor, 0, (hipStream_t)stream));
}

int llmint8_export_rows(const int8_t* Xq, int s, int h, int8_t* X_i8_rowmajor, llmint8_stream_t stream)
{
    if (!Xq || !X_i8_rowmajor || s < 1 || h < 1 || misaligned(Xq, 16)) return LLMINT8_INVALID_ARG;
    return hip_status(launch_export_tiled(Xq, s, h, X_i8_rowmajor, 1, (hipStream_t)stream));
}

}  // extern "C"
