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


// ---- pairwise path on the matrix cores --------------------------------------------------------------------------
// The similarity equation taken literally: C = E_v E_t^T (every window token against every text token), then
// c_k = 1/(N |w_k|) sum_j C[k,j] / |t_j|.  One workgroup owns 128 visual rows of one sequence and walks the text
// tokens in column tiles of 128; per column tile a classic LDS-tiled GEMM over D in steps of 32
// (v_mfma_f32_16x16x32 bf16/f16, four wavefronts as 2x2, 64x64 per wavefront), whose epilogue multiplies by
// 1/|t_j| and reduces over the columns, so C never leaves the registers.  |w_k|^2 comes from the A tiles on their
// way to LDS during the first column tile.  Reductions have a fixed order: results are deterministic.
typedef float floatx4s __attribute__((ext_vector_type(4)));
typedef _Float16 half8s __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x8s __attribute__((ext_vector_type(8)));

template <bool BF>
__device__ __forceinline__ floatx4s mfma_s(const uint4& a, const uint4& b, floatx4s c)
{
    if constexpr (BF)
        return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8s, a), __builtin_bit_cast(bf16x8s, b), c, 0, 0, 0);
    else
        return __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(half8s, a), __builtin_bit_cast(half8s, b), c, 0, 0, 0);
}

template <bool BF>
__device__ __forceinline__ float sumsq8(const uint4& u)
{
    const uint32_t w[4] = {u.x, u.y, u.z, u.w};
    float s = 0.f;
#pragma unroll
    for (int k = 0; k < 4; k++) {
        const float a = BF ? __uint_as_float(w[k] << 16) : wq_f16_bits_to_float(w[k] & 0xFFFFu);
        const float b = BF ? __uint_as_float(w[k] & 0xFFFF0000u) : wq_f16_bits_to_float(w[k] >> 16);
        s = fmaf(a, a, s);
        s = fmaf(b, b, s);
    }
    return s;
}

constexpr int SG_PITCH = 40;     // 16-bit elements per LDS row: 32 of the k-step + 8 of padding (80 bytes)

template <bool BF>
__global__ __launch_bounds__(256) void k_pair_mfma(const uint16_t* __restrict__ vis, const uint16_t* __restrict__ txt,
                                                   const float* __restrict__ inv_tnorm, int D,
                                                   const int32_t* __restrict__ vis_off, const int32_t* __restrict__ txt_off,
                                                   float* __restrict__ tok_score)
{
    __shared__ __align__(16) uint16_t sA[128 * SG_PITCH];
    __shared__ __align__(16) uint16_t sB[128 * SG_PITCH];
    __shared__ float sW[128];          // 1/|t_j| of the column tile (0 past the end)
    __shared__ float sR[2][128];       // row sums, one array per column half of the wavefront grid
    __shared__ float sN[128];          // |w_k|^2
    const int b = blockIdx.y;
    const int m0 = vis_off[b], M = vis_off[b + 1] - m0;
    const int n0 = txt_off[b], N = txt_off[b + 1] - n0;
    const int row0 = blockIdx.x * 128;
    if (row0 >= M) return;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wr = wave >> 1, wc = wave & 1;             // 2 x 2 wavefronts, 64 x 64 each
    const int lj = lane >> 4, lm = lane & 15;
    // global -> LDS staging: 128 rows x 64 bytes = 512 pieces of 16 bytes, two per thread (pieces tid, tid + 256)
    const int pr0 = tid >> 2, pp = tid & 3;              // row and 16-byte part of piece tid; piece tid+256: row + 64
    const int ra0 = min(row0 + pr0, M - 1), ra1 = min(row0 + pr0 + 64, M - 1);      // rows past the end re-read the last
    const uint16_t* pa0 = vis + ((int64_t)m0 + ra0) * D + pp * 8;
    const uint16_t* pa1 = vis + ((int64_t)m0 + ra1) * D + pp * 8;
    if (tid < 128) {
        sR[0][tid] = 0.f;
        sR[1][tid] = 0.f;
    }
    float nsq0 = 0.f, nsq1 = 0.f;
    const int ksteps = D / 32;
    for (int c0 = 0; c0 < N; c0 += 128) {
        const int rb0 = min(c0 + pr0, N - 1), rb1 = min(c0 + pr0 + 64, N - 1);
        const uint16_t* pb0 = txt + ((int64_t)n0 + rb0) * D + pp * 8;
        const uint16_t* pb1 = txt + ((int64_t)n0 + rb1) * D + pp * 8;
        __syncthreads();                                  // previous tile's epilogue has read sW
        if (tid < 128) sW[tid] = (c0 + tid < N) ? inv_tnorm[n0 + c0 + tid] : 0.f;
        floatx4s acc[4][4];
#pragma unroll
        for (int i = 0; i < 4; i++)
#pragma unroll
            for (int k = 0; k < 4; k++) acc[i][k] = floatx4s{0.f, 0.f, 0.f, 0.f};
        uint4 ga0 = *reinterpret_cast<const uint4*>(pa0), ga1 = *reinterpret_cast<const uint4*>(pa1);
        uint4 gb0 = *reinterpret_cast<const uint4*>(pb0), gb1 = *reinterpret_cast<const uint4*>(pb1);
        for (int ks = 0; ks < ksteps; ks++) {
            __syncthreads();                              // everyone is done reading the previous k-step's tiles
            *reinterpret_cast<uint4*>(&sA[pr0 * SG_PITCH + pp * 8]) = ga0;
            *reinterpret_cast<uint4*>(&sA[(pr0 + 64) * SG_PITCH + pp * 8]) = ga1;
            *reinterpret_cast<uint4*>(&sB[pr0 * SG_PITCH + pp * 8]) = gb0;
            *reinterpret_cast<uint4*>(&sB[(pr0 + 64) * SG_PITCH + pp * 8]) = gb1;
            if (c0 == 0) {
                nsq0 += sumsq8<BF>(ga0);
                nsq1 += sumsq8<BF>(ga1);
            }
            __syncthreads();
            if (ks + 1 < ksteps) {                        // next k-step's pieces fly while this one is multiplied
                const int o = (ks + 1) * 32;
                ga0 = *reinterpret_cast<const uint4*>(pa0 + o);
                ga1 = *reinterpret_cast<const uint4*>(pa1 + o);
                gb0 = *reinterpret_cast<const uint4*>(pb0 + o);
                gb1 = *reinterpret_cast<const uint4*>(pb1 + o);
            }
            uint4 fa[4], fb[4];
#pragma unroll
            for (int i = 0; i < 4; i++) {
                fa[i] = *reinterpret_cast<const uint4*>(&sA[(wr * 64 + i * 16 + lm) * SG_PITCH + lj * 8]);
                fb[i] = *reinterpret_cast<const uint4*>(&sB[(wc * 64 + i * 16 + lm) * SG_PITCH + lj * 8]);
            }
#pragma unroll
            for (int i = 0; i < 4; i++)
#pragma unroll
                for (int k = 0; k < 4; k++) acc[i][k] = mfma_s<BF>(fa[i], fb[k], acc[i][k]);
        }
        // epilogue: lane holds rows 4*lj + e of row tile i, column lm of column tile k
#pragma unroll
        for (int i = 0; i < 4; i++) {
            float rs[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int k = 0; k < 4; k++) {
                const float w = sW[wc * 64 + k * 16 + lm];
#pragma unroll
                for (int e = 0; e < 4; e++) rs[e] = fmaf(acc[i][k][e], w, rs[e]);
            }
#pragma unroll
            for (int e = 0; e < 4; e++) {
                float v = rs[e];
                v += __shfl_xor(v, 1, 64);
                v += __shfl_xor(v, 2, 64);
                v += __shfl_xor(v, 4, 64);
                v += __shfl_xor(v, 8, 64);
                if (lm == 0) sR[wc][wr * 64 + i * 16 + 4 * lj + e] += v;     // one writer per (column half, row)
            }
        }
    }
    // |w_k|^2: the four threads that staged a row hold its four 16-byte parts of every k-step
    nsq0 += __shfl_xor(nsq0, 1, 64);
    nsq0 += __shfl_xor(nsq0, 2, 64);
    nsq1 += __shfl_xor(nsq1, 1, 64);
    nsq1 += __shfl_xor(nsq1, 2, 64);
    if (pp == 0) {
        sN[pr0] = nsq0;
        sN[pr0 + 64] = nsq1;
    }
    __syncthreads();
    if (tid < 128 && row0 + tid < M) {
        const float r = sR[0][tid] + sR[1][tid], nn = sN[tid];
        tok_score[m0 + row0 + tid] = (nn > 0.f && N > 0) ? r / (sqrtf(nn) * (float)N) : 0.f;
    }
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
    if (algo == WQ_SCORE_PAIRWISE_MFMA) {
        if (D % 32 != 0) return wq_fail(ctx, WQ_ERR_UNSUPPORTED, "the matrix-core scoring path needs D %% 32 == 0");
        if ((reinterpret_cast<uintptr_t>(vis) | reinterpret_cast<uintptr_t>(txt)) % 16 != 0)
            return wq_fail(ctx, WQ_ERR_ARG, "embeddings must be 16-byte aligned");
        char* ws = ctx->ws + WQ_WS_HEADER;
        float* inv_norm = reinterpret_cast<float*>(ws);
        ws += wq_align256(sizeof(float) * (size_t)(total_txt > 0 ? total_txt : 1));
        ws += wq_align256(sizeof(float) * (size_t)B * D);
        float* tok_score = reinterpret_cast<float*>(ws);
        hipStream_t st = ctx->stream;
        const uint16_t* v16 = static_cast<const uint16_t*>(vis);
        const uint16_t* t16 = static_cast<const uint16_t*>(txt);
        if (total_txt > 0) {
            if (dtype == WQ_BF16)
                hipLaunchKernelGGL((k_text_norm<__hip_bfloat16, true>), dim3((unsigned)((total_txt + 3) / 4)), dim3(256), 0, st,
                                   static_cast<const __hip_bfloat16*>(txt), D, total_txt, inv_norm);
            else
                hipLaunchKernelGGL((k_text_norm<__half, true>), dim3((unsigned)((total_txt + 3) / 4)), dim3(256), 0, st,
                                   static_cast<const __half*>(txt), D, total_txt, inv_norm);
        }
        if (total_vis > 0) {
            // any one sequence has at most total_vis rows: row tiles past a sequence's end return at once
            const dim3 grid((unsigned)((total_vis + 127) / 128), B);
            if (dtype == WQ_BF16)
                hipLaunchKernelGGL(k_pair_mfma<true>, grid, dim3(256), 0, st, v16, t16, inv_norm, D, vis_off, txt_off, tok_score);
            else
                hipLaunchKernelGGL(k_pair_mfma<false>, grid, dim3(256), 0, st, v16, t16, inv_norm, D, vis_off, txt_off, tok_score);
        }
        hipLaunchKernelGGL(k_window_mean, dim3((unsigned)((total_win + 3) / 4)), dim3(256), 0, st, tok_score, B, vis_off, txt_off,
                           win_size, win_off, total_win, scores);
        WQ_HIP_CHECK(ctx, hipGetLastError());
        return WQ_OK;
    }
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
