// Internal declarations shared by the translation units of libwq (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <hip/hip_bf16.h>
#include <hip/hip_fp16.h>
#include <stdarg.h>
#include <stdint.h>
#include <stdio.h>

#include "../../include/wq.h"
#include "../../include/wq_measure.h"

struct wq_ctx {
    hipStream_t stream;
    char* ws;            // device workspace
    size_t ws_bytes;
    bool owns_ws;
    bool timing;                 // record an event pair around the main decode kernel of every call
    hipEvent_t ev[2 * 64];       // ring of WQ_TIMING_RING pairs (created by wq_decode_timing)
    uint64_t ev_calls;           // decode calls timed so far
    char err[256];
};

constexpr size_t WQ_WS_HEADER = 16384; // zero-initialised: status word (first 256 bytes), then the decode kernel's arrival counters
constexpr int WQ_ARRIVE_STRIDE = 16;   // 32-bit words between arrival counters (one 64-byte piece each)
constexpr int WQ_MAX_ARRIVE = (16384 - 256) / (4 * WQ_ARRIVE_STRIDE);
constexpr int WQ_DECODE_FLAGS = WQ_DECODE_PARTIALS_ONLY | WQ_DECODE_FIXED_SHARES | WQ_DECODE_BY_LENGTH | WQ_DECODE_SEPARATE_MERGE;
constexpr int WQ_TIMING_RING = 64;
constexpr int WQ_MAX_REP = 8;          // query heads per KV head
constexpr int WQ_MAX_FUSED_SPLITS = 64; // splits that the decode kernel merges itself (one per lane of a wavefront)
// wall time of one 32-token block of the 2-, 4-, 8- and 16-bit class in the decode kernel, relative to each other
// (measured on MI355X with the whole chip streaming): the fixed shares of the token axis are balanced by it
#ifndef WQ_COSTS
#define WQ_COSTS 100, 130, 230, 500
#endif
constexpr int WQ_BLOCK_COST[4] = {WQ_COSTS};
constexpr int WQ_MAX_WINDOWS = 8192;   // windows per sequence handled by the ranking kernel

inline int wq_fail(wq_ctx* ctx, int code, const char* fmt, ...)
{
    if (ctx) {
        va_list ap;
        va_start(ap, fmt);
        vsnprintf(ctx->err, sizeof(ctx->err), fmt, ap);
        va_end(ap);
    }
    return code;
}

#define WQ_HIP_CHECK(ctx, expr)                                                              \
    do {                                                                                     \
        hipError_t e_ = (expr);                                                              \
        if (e_ != hipSuccess) return wq_fail(ctx, WQ_ERR_HIP, "%s: %s", #expr, hipGetErrorString(e_)); \
    } while (0)

inline size_t wq_align256(size_t x) { return (x + 255) & ~size_t(255); }
inline uint32_t* wq_status_ptr(wq_ctx* ctx) { return reinterpret_cast<uint32_t*>(ctx->ws); }

// element loads -> float (exact for all three storage types)
__device__ __forceinline__ float wq_ld(const float* p, int64_t i) { return p[i]; }
__device__ __forceinline__ float wq_ld(const __hip_bfloat16* p, int64_t i)
{
    return __uint_as_float(uint32_t(reinterpret_cast<const uint16_t*>(p)[i]) << 16);
}
__device__ __forceinline__ float wq_ld(const __half* p, int64_t i) { return __half2float(p[i]); }

__device__ __forceinline__ float wq_bf16_bits_to_float(uint32_t h) { return __uint_as_float(h << 16); }
__device__ __forceinline__ float wq_f16_bits_to_float(uint32_t h)
{
    return __half2float(__ushort_as_half(static_cast<unsigned short>(h)));
}

// 8 consecutive elements of a row as floats (16-byte loads for the 16-bit types, 2 x 16 for fp32)
__device__ __forceinline__ void wq_ld8(const float* p, float* x)
{
    const float4 a = *reinterpret_cast<const float4*>(p), b = *reinterpret_cast<const float4*>(p + 4);
    x[0] = a.x, x[1] = a.y, x[2] = a.z, x[3] = a.w, x[4] = b.x, x[5] = b.y, x[6] = b.z, x[7] = b.w;
}
__device__ __forceinline__ void wq_ld8(const __hip_bfloat16* p, float* x)
{
    const uint4 u = *reinterpret_cast<const uint4*>(p);
    const uint32_t w[4] = {u.x, u.y, u.z, u.w};
#pragma unroll
    for (int k = 0; k < 4; k++) {
        x[2 * k] = __uint_as_float(w[k] << 16);
        x[2 * k + 1] = __uint_as_float(w[k] & 0xFFFF0000u);
    }
}
__device__ __forceinline__ void wq_ld8(const __half* p, float* x)
{
    const uint4 u = *reinterpret_cast<const uint4*>(p);
    const uint32_t w[4] = {u.x, u.y, u.z, u.w};
#pragma unroll
    for (int k = 0; k < 4; k++) {
        x[2 * k] = wq_f16_bits_to_float(w[k] & 0xFFFFu);
        x[2 * k + 1] = wq_f16_bits_to_float(w[k] >> 16);
    }
}

// first b in [0,B) with off[b+1] > x  (off ascending, off[0] <= x < off[B] assumed)
__device__ __forceinline__ int wq_find_seq(const int32_t* off, int B, int64_t x)
{
    int lo = 0, hi = B;            // invariant: off[lo] <= x < off[hi]
    while (hi - lo > 1) {
        int mid = (lo + hi) >> 1;
        if (off[mid] <= x) lo = mid; else hi = mid;
    }
    return lo;
}

// launchers (one per stage), defined next to their kernels
int wq_launch_scores(wq_ctx* ctx, const void* vis, const void* txt, int dtype, int B, int D, const int32_t* vis_off,
                     const int32_t* txt_off, const int32_t* win_size, const int32_t* win_off, int64_t total_vis,
                     int64_t total_txt, int64_t total_win, int algo, float* scores);
int wq_launch_assign(wq_ctx* ctx, const float* scores, int B, const int32_t* win_off, int max_windows, int mode,
                     const int32_t* quota, const float* thresholds, int top_bits, int pin_first, uint8_t* bits,
                     int32_t* perm, int32_t* seg_windows);
int wq_launch_vote(wq_ctx* ctx, const uint8_t* bits_in, int B, const int32_t* win_off, int max_windows, uint8_t* bits_out, int32_t* perm,
                   int32_t* seg_windows);
int wq_launch_validate(wq_ctx* ctx, int B, const int32_t* win_off, int max_windows, const int32_t* perm, const int32_t* seg_windows);
int wq_launch_quantize(wq_ctx* ctx, const void* K, const void* V, int dtype, int B, const int32_t* kv_off,
                       const int32_t* win_size, const int32_t* win_off, const int32_t* perm,
                       const int32_t* seg_windows, int64_t total_rows, const wq_packed_kv* out);
int wq_launch_append(wq_ctx* ctx, const void* k_new, const void* v_new, int dtype, int B, const wq_packed_kv* kv);
int wq_launch_dequantize(wq_ctx* ctx, int B, const wq_packed_kv* src, const wq_packed_kv* dst);
int wq_launch_decode(wq_ctx* ctx, const void* q, int q_dtype, int B, int Hq, const wq_packed_kv* kv, float sm_scale,
                     int num_splits, int algo, float* out, float* lse, const void* k_new = nullptr, const void* v_new = nullptr,
                     int64_t longest_tokens = 0);
bool wq_decode_can_append(int q_dtype, int B, int Hq, const wq_packed_kv* kv, int num_splits, int algo, int new_dtype);
size_t wq_decode_ws_bytes(int B, int Hq, int hd, int splits);
size_t wq_scores_ws_bytes(int B, int64_t total_vis, int64_t total_txt, int D);
