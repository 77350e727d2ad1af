// a1: window/text similarity (Sec. 3.2.1, similarity equation).
//
// Pooled path: by linearity the mean of all pairwise cosines of a window equals
//     (mean_j t_j/|t_j|) . (mean_k w_k/|w_k|),
// so every embedding row is read exactly once: the kernels are bound by HBM bandwidth.
//   k_text_norm   one wavefront per text token  -> 1/|t_j|                       (0 for a zero row)
//   k_text_mean   thread per channel            -> tbar[b][d] = 1/N sum_j t_j[d]/|t_j|
//   k_token_score one wavefront per visual row  -> c_k = (w_k . tbar) / |w_k|    (0 for a zero row)
//   k_window_mean one wavefront per window      -> score = 1/S sum_k c_k, fixed order
// All accumulation is fp32 and every reduction has a fixed order (no atomics): results are deterministic.
#include "wq_internal.h"

namespace {

constexpr int WAVE = 64;

__device__ __forceinline__ float wave_sum(float v)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, WAVE);
    return v;
}

// VEC: rows are read 8 elements per lane (needs D % 8 == 0); otherwise element by element.
template <typename T, bool VEC>
__global__ __launch_bounds__(256) void k_text_norm(const T* __restrict__ txt, int D, int64_t total_txt,
                                                   float* __restrict__ inv_norm)
{
    int64_t row = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (row >= total_txt) return;
    int lane = threadIdx.x & 63;
    const T* p = txt + row * D;
    float ss = 0.f;
    if (VEC) {
        for (int d = lane * 8; d < D; d += WAVE * 8) {
            float x[8];
            wq_ld8(p + d, x);
#pragma unroll
            for (int k = 0; k < 8; k++) ss = fmaf(x[k], x[k], ss);
        }
    } else {
        for (int d = lane; d < D; d += WAVE) {
            float x = wq_ld(p, d);
            ss = fmaf(x, x, ss);
        }
    }
    ss = wave_sum(ss);
    if (lane == 0) inv_norm[row] = ss > 0.f ? 1.0f / sqrtf(ss) : 0.f;
}

// tbar[b][d] = 1/N sum_j t_j[d]/|t_j|.  VEC: thread = (8 columns, one of 8 token slices), slices merged in LDS in
// slice order; otherwise one thread per column.
template <typename T, bool VEC>
__global__ __launch_bounds__(256) void k_text_mean(const T* __restrict__ txt, const float* __restrict__ inv_norm, int D,
                                                   const int32_t* __restrict__ txt_off, float* __restrict__ tbar)
{
    const int b = blockIdx.y;
    const int j0 = txt_off[b], j1 = txt_off[b + 1];
    if (VEC) {
        __shared__ float s_acc[8][32][9];
        const int cc = threadIdx.x & 31, ts = threadIdx.x >> 5;
        const int d0 = (blockIdx.x * 32 + cc) * 8;
        float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
        if (d0 < D)
            for (int j = j0 + ts; j < j1; j += 8) {
                float x[8];
                wq_ld8(txt + (int64_t)j * D + d0, x);
                const float w = inv_norm[j];
#pragma unroll
                for (int k = 0; k < 8; k++) acc[k] = fmaf(x[k], w, acc[k]);
            }
#pragma unroll
        for (int k = 0; k < 8; k++) s_acc[ts][cc][k] = acc[k];
        __syncthreads();
        const int c2 = threadIdx.x >> 3, k2 = threadIdx.x & 7;      // 32 chunks x 8 columns
        const int d = (blockIdx.x * 32 + c2) * 8 + k2;
        if (d < D) {
            float s = 0.f;
#pragma unroll
            for (int t = 0; t < 8; t++) s += s_acc[t][c2][k2];
            tbar[(int64_t)b * D + d] = j1 > j0 ? s / (float)(j1 - j0) : 0.f;
        }
    } else {
        int d = blockIdx.x * 256 + threadIdx.x;
        if (d >= D) return;
        float acc = 0.f;
        for (int j = j0; j < j1; j++) acc = fmaf(wq_ld(txt, (int64_t)j * D + d), inv_norm[j], acc);
        tbar[(int64_t)b * D + d] = j1 > j0 ? acc / (float)(j1 - j0) : 0.f;
    }
}

// c_k = (w_k . tbar) / |w_k|.  VEC: one wavefront takes 4 consecutive rows so that each 32-byte piece of the pooled
// text vector is loaded once per 4 rows; 16 bytes of every row per lane and iteration.
template <typename T, bool VEC>
__global__ __launch_bounds__(256) void k_token_score(const T* __restrict__ vis, const float* __restrict__ tbar, int D, int B,
                                                     const int32_t* __restrict__ vis_off, int64_t total_vis,
                                                     float* __restrict__ tok_score)
{
    const int lane = threadIdx.x & 63;
    if (VEC) {
        const int64_t row0 = ((int64_t)blockIdx.x * 4 + (threadIdx.x >> 6)) * 4;
        if (row0 >= total_vis) return;
        int bs[4];
        const T* p[4];
#pragma unroll
        for (int r = 0; r < 4; r++) {
            const int64_t row = row0 + r < total_vis ? row0 + r : total_vis - 1;
            bs[r] = wq_find_seq(vis_off, B, row);
            p[r] = vis + row * D;
        }
        const bool same = bs[0] == bs[3];          // rows are ordered by sequence: all four share one text vector
        float ss[4] = {0.f, 0.f, 0.f, 0.f}, dt[4] = {0.f, 0.f, 0.f, 0.f};
        for (int d = lane * 8; d < D; d += WAVE * 8) {
            float t[8];
            wq_ld8(tbar + (int64_t)bs[0] * D + d, t);
#pragma unroll
            for (int r = 0; r < 4; r++) {
                float x[8], tr[8];
                wq_ld8(p[r] + d, x);
                if (!same && bs[r] != bs[0]) wq_ld8(tbar + (int64_t)bs[r] * D + d, tr);
#pragma unroll
                for (int k = 0; k < 8; k++) {
                    const float tk = (!same && bs[r] != bs[0]) ? tr[k] : t[k];
                    ss[r] = fmaf(x[k], x[k], ss[r]);
                    dt[r] = fmaf(x[k], tk, dt[r]);
                }
            }
        }
#pragma unroll
        for (int r = 0; r < 4; r++) {
            const float s = wave_sum(ss[r]), d2 = wave_sum(dt[r]);
            if (lane == 0 && row0 + r < total_vis) tok_score[row0 + r] = s > 0.f ? d2 / sqrtf(s) : 0.f;
        }
    } else {
        int64_t row = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
        if (row >= total_vis) return;
        int b = wq_find_seq(vis_off, B, row);
        const T* p = vis + row * D;
        const float* t = tbar + (int64_t)b * D;
        float ss = 0.f, dt = 0.f;
        for (int d = lane; d < D; d += WAVE) {
            float x = wq_ld(p, d);
            ss = fmaf(x, x, ss);
            dt = fmaf(x, t[d], dt);
        }
        ss = wave_sum(ss);
        dt = wave_sum(dt);
        if (lane == 0) tok_score[row] = ss > 0.f ? dt / sqrtf(ss) : 0.f;
    }
}

__global__ __launch_bounds__(256) void k_window_mean(const float* __restrict__ tok_score, int B,
                                                     const int32_t* __restrict__ vis_off, const int32_t* __restrict__ txt_off,
                                                     const int32_t* __restrict__ win_size, const int32_t* __restrict__ win_off,
                                                     int64_t total_win, float* __restrict__ scores)
{
    int64_t w = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (w >= total_win) return;
    int lane = threadIdx.x & 63;
    int b = wq_find_seq(win_off, B, w);
    int S = win_size[b];
    int64_t r0 = (int64_t)vis_off[b] + (w - win_off[b]) * S;
    float acc = 0.f;
    for (int k = lane; k < S; k += WAVE) acc += tok_score[r0 + k];
    acc = wave_sum(acc);
    if (lane == 0) scores[w] = (S > 0 && txt_off[b + 1] > txt_off[b]) ? acc / (float)S : 0.f;
}

template <typename T, bool VEC>
int run_pooled(wq_ctx* ctx, const void* vis_, const void* txt_, int B, int D, const int32_t* vis_off, const int32_t* txt_off,
               const int32_t* win_size, const int32_t* win_off, int64_t total_vis, int64_t total_txt, int64_t total_win,
               float* scores)
{
    const T* vis = static_cast<const T*>(vis_);
    const T* txt = static_cast<const T*>(txt_);
    char* ws = ctx->ws + WQ_WS_HEADER;
    float* inv_norm = reinterpret_cast<float*>(ws);
    ws += wq_align256(sizeof(float) * (size_t)(total_txt > 0 ? total_txt : 1));
    float* tbar = reinterpret_cast<float*>(ws);
    ws += wq_align256(sizeof(float) * (size_t)B * D);
    float* tok_score = reinterpret_cast<float*>(ws);
    hipStream_t st = ctx->stream;
    if (total_txt > 0)
        hipLaunchKernelGGL((k_text_norm<T, VEC>), dim3((unsigned)((total_txt + 3) / 4)), dim3(256), 0, st, txt, D, total_txt, inv_norm);
    hipLaunchKernelGGL((k_text_mean<T, VEC>), dim3((D + 255) / 256, B), dim3(256), 0, st, txt, inv_norm, D, txt_off, tbar);
    if (total_vis > 0) {
        const int64_t rows_per_block = VEC ? 16 : 4;
        hipLaunchKernelGGL((k_token_score<T, VEC>), dim3((unsigned)((total_vis + rows_per_block - 1) / rows_per_block)), dim3(256), 0, st,
                           vis, tbar, D, B, vis_off, total_vis, tok_score);
    }
    hipLaunchKernelGGL(k_window_mean, dim3((unsigned)((total_win + 3) / 4)), dim3(256), 0, st, tok_score, B, vis_off, txt_off,
                       win_size, win_off, total_win, scores);
    WQ_HIP_CHECK(ctx, hipGetLastError());
    return WQ_OK;
}

}  // namespace

size_t wq_scores_ws_bytes(int B, int64_t total_vis, int64_t total_txt, int D)
{
    if (B <= 0 || D <= 0) return 0;
    return wq_align256(sizeof(float) * (size_t)(total_txt > 0 ? total_txt : 1)) + wq_align256(sizeof(float) * (size_t)B * D) +
           wq_align256(sizeof(float) * (size_t)(total_vis > 0 ? total_vis : 1));
}

int wq_launch_scores(wq_ctx* ctx, const void* vis, const void* txt, int dtype, int B, int D, const int32_t* vis_off,
                     const int32_t* txt_off, const int32_t* win_size, const int32_t* win_off, int64_t total_vis,
                     int64_t total_txt, int64_t total_win, int algo, float* scores)
{
    if (algo == WQ_SCORE_PAIRWISE_MFMA)
        return wq_fail(ctx, WQ_ERR_UNSUPPORTED, "matrix-core scoring path is not built yet");
    // 16-byte row pieces need D % 8 == 0 and 16-byte aligned bases (rows then stay aligned for every element type)
    const bool vec = D % 8 == 0 && (reinterpret_cast<uintptr_t>(vis) | reinterpret_cast<uintptr_t>(txt)) % 16 == 0;
#define WQ_RUN(T)                                                                                                         \
    (vec ? run_pooled<T, true>(ctx, vis, txt, B, D, vis_off, txt_off, win_size, win_off, total_vis, total_txt, total_win, scores) \
         : run_pooled<T, false>(ctx, vis, txt, B, D, vis_off, txt_off, win_size, win_off, total_vis, total_txt, total_win, scores))
    switch (dtype) {
        case WQ_F32: return WQ_RUN(float);
        case WQ_BF16: return WQ_RUN(__hip_bfloat16);
        default: return WQ_RUN(__half);
    }
#undef WQ_RUN
}

// ---- measurement probes (not part of the method): plain streaming kernels of known size -----------------------
namespace {

__global__ __launch_bounds__(256) void k_probe_read(const uint4* __restrict__ src, int64_t n16, uint32_t* __restrict__ sink)
{
    uint32_t acc = 0;
    const int64_t stride = (int64_t)gridDim.x * 256;
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n16; i += stride) {
        uint4 v = src[i];
        acc ^= v.x ^ v.y ^ v.z ^ v.w;
    }
    if (acc == 0x9E3779B9u) sink[0] = acc;   // practically never true; keeps the loads alive
}

__global__ __launch_bounds__(256) void k_probe_copy(const uint4* __restrict__ src, uint4* __restrict__ dst, int64_t n16)
{
    const int64_t stride = (int64_t)gridDim.x * 256;
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n16; i += stride) dst[i] = src[i];
}

}  // namespace

extern "C" int wq_probe_stream(wq_ctx* ctx, const void* src, void* dst, int64_t bytes, int blocks)
{
    if (!ctx || !src || bytes < 16 || blocks <= 0) return WQ_ERR_ARG;
    const int64_t n16 = bytes / 16;
    if (dst)
        hipLaunchKernelGGL(k_probe_copy, dim3(blocks), dim3(256), 0, ctx->stream, static_cast<const uint4*>(src),
                           static_cast<uint4*>(dst), n16);
    else
        hipLaunchKernelGGL(k_probe_read, dim3(blocks), dim3(256), 0, ctx->stream, static_cast<const uint4*>(src), n16,
                           wq_status_ptr(ctx) + 8);
    WQ_HIP_CHECK(ctx, hipGetLastError());
    return WQ_OK;
}
