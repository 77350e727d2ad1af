// a2: bit-width per window and the stable class order (Sec. 3.2.1 threshold rule, Sec. 3.2.2 first-window
// pin, Alg. 2 prefill loop; rank/quota rule).  At most WQ_MAX_WINDOWS windows per sequence.
//   k_assign both steps below in one workgroup per sequence (sequences of up to ASSIGN_ONE_LAUNCH windows)
//   k_rank   widths: ranks come from counting (rank_i = #{j : s_j > s_i or (s_j == s_i and j < i)}), which needs no
//            sort and is exact on fp32 compares; a workgroup per 64 windows
//   k_order  class positions from counting equal-class predecessors; a workgroup per sequence
// Integer-only results, so the output is bit-exact by construction.
#include "wq_internal.h"

namespace {

__device__ __forceinline__ int class_of(int bits) { return bits == 2 ? 0 : (bits == 4 ? 1 : (bits == 8 ? 2 : 3)); }

constexpr int ASSIGN_THREADS = 1024;

// Widths of one sequence are in s_bits: writes them out, counts the classes and lists the windows class by class
// (2-, 4-, 8-, 16-bit), each class in index order.  A window's place is its class's first place plus the number of
// earlier windows of its class: counted per chunk of 64 windows with a ballot per class (the earlier lanes of the
// wavefront), plus the classes' counts over the chunks before it (s_chunk, made a running sum by four lanes).
constexpr int ASSIGN_CHUNKS = WQ_MAX_WINDOWS / 64;
__device__ __forceinline__ void emit_class_order(const uint8_t* s_bits, int* s_cnt, int (*s_chunk)[4], int W, int w0, int b,
                                                 uint8_t* __restrict__ bits, int32_t* __restrict__ perm, int32_t* __restrict__ seg_windows)
{
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, nwaves = ASSIGN_THREADS / 64;
    const int chunks = (W + 63) >> 6;
    const unsigned long long earlier = (1ull << lane) - 1ull;
    for (int ch = wave; ch < chunks; ch += nwaves) {
        const int i = ch * 64 + lane;
        const int c = i < W ? class_of(s_bits[i]) : -1;
        if (i < W) bits[w0 + i] = s_bits[i];
#pragma unroll
        for (int k = 0; k < 4; k++) {
            const unsigned long long m = __ballot(c == k);
            if (lane == 0) s_chunk[ch][k] = __popcll(m);
        }
    }
    __syncthreads();
    if (tid < 4) {                               // a class's count, and its chunks' counts as sums over the chunks before
        int run = 0;
        for (int ch = 0; ch < chunks; ch++) {
            const int n = s_chunk[ch][tid];
            s_chunk[ch][tid] = run;
            run += n;
        }
        s_cnt[tid] = run;
        seg_windows[4 * b + tid] = run;
    }
    __syncthreads();
    for (int ch = wave; ch < chunks; ch += nwaves) {
        const int i = ch * 64 + lane;
        const int c = i < W ? class_of(s_bits[i]) : -1;
        int pos = 0;
#pragma unroll
        for (int k = 0; k < 4; k++) {
            const unsigned long long m = __ballot(c == k);
            if (c == k) pos += s_chunk[ch][k] + __popcll(m & earlier);
            if (c > k) pos += s_cnt[k];          // (accumulates the first places of the classes before c)
        }
        if (i < W) perm[w0 + pos] = i;
    }
}

// Batch-shared configuration (Sec. 3.2.3, last paragraph): one workgroup per sequence; every lane takes window
// positions of that sequence and counts, over the sequences that have the position, how often each width occurs.
// Most votes win, the wider width on a tie.
__global__ __launch_bounds__(ASSIGN_THREADS) void k_vote(const uint8_t* __restrict__ bits_in, int B, const int32_t* __restrict__ win_off,
                                                         uint8_t* __restrict__ bits, int32_t* __restrict__ perm,
                                                         int32_t* __restrict__ seg_windows, int max_windows, uint32_t* __restrict__ status)
{
    __shared__ __align__(16) uint8_t s_bits[WQ_MAX_WINDOWS + 4];
    __shared__ int s_cnt[4];
    __shared__ int s_chunk[ASSIGN_CHUNKS][4];
    const int b = blockIdx.x;
    const int w0 = win_off[b];
    int W = win_off[b + 1] - w0;
    const int tid = threadIdx.x;
    if (W > max_windows) {                        // reported; only the positions inside the caller's bound are voted on
        if (tid == 0) atomicOr(status, WQ_DEV_TOO_MANY_WINDOWS);
        W = max_windows;
    }
    const int W4 = (W + 3) & ~3;
    if (tid < 4) s_cnt[tid] = 0;
    for (int p = tid; p < W4; p += ASSIGN_THREADS) {
        int votes[4] = {0, 0, 0, 0};
        if (p < W) {
            for (int o = 0; o < B; o++) {
                const int o0 = win_off[o];
                if (win_off[o + 1] - o0 > p) votes[class_of(bits_in[o0 + p])]++;
            }
        }
        int best = 0;
#pragma unroll
        for (int c = 1; c < 4; c++) best = votes[c] >= votes[best] ? c : best;     // >= : the wider width on a tie
        s_bits[p] = p < W ? (uint8_t)(best == 0 ? 2 : (best == 1 ? 4 : (best == 2 ? 8 : 16))) : (uint8_t)0;
    }
    __syncthreads();                 // every lane is done reading bits_in before anything is written (it may alias bits)
    emit_class_order(s_bits, s_cnt, s_chunk, W, w0, b, bits, perm, seg_windows);
}

// Widths and class order of a sequence in one workgroup: for sequences of a few hundred windows, where the second
// launch of the other way costs more than the counting that it spreads over the chip.
__global__ __launch_bounds__(ASSIGN_THREADS) void k_assign(const float* __restrict__ scores, const int32_t* __restrict__ win_off, int mode,
                                                           const int32_t* __restrict__ quota, const float* __restrict__ thresholds,
                                                           int top_bits, int pin_first, uint8_t* __restrict__ bits,
                                                           int32_t* __restrict__ perm, int32_t* __restrict__ seg_windows,
                                                           int max_windows, uint32_t* __restrict__ status)
{
    // keys and widths are read four at a time in the counting loops; both arrays are padded to a multiple of four
    // (keys with -inf, which no key is smaller than and which never counts as an earlier equal; widths with 0)
    __shared__ __align__(16) float s_key[WQ_MAX_WINDOWS + 4];
    __shared__ __align__(16) uint8_t s_bits[WQ_MAX_WINDOWS + 4];
    __shared__ int s_cnt[4];
    __shared__ int s_chunk[ASSIGN_CHUNKS][4];
    const int b = blockIdx.x;
    const int w0 = win_off[b];
    int W = win_off[b + 1] - w0;
    const int tid = threadIdx.x;
    if (W > max_windows) {                        // more windows than the caller's bound (itself at most WQ_MAX_WINDOWS): reported,
        if (tid == 0) atomicOr(status, WQ_DEV_TOO_MANY_WINDOWS);      // and only the windows inside the bound are assigned
        W = max_windows;
    }
    const int W4 = (W + 3) & ~3;
    if (tid < 4) s_cnt[tid] = 0;
    for (int i = tid; i < W4; i += ASSIGN_THREADS) {
        float s = i < W ? scores[w0 + i] : -INFINITY;
        s_key[i] = (s != s) ? -INFINITY : s;
        if (i >= W) s_bits[i] = 0;
    }
    __syncthreads();

    if (mode == WQ_MODE_THRESHOLD) {
        float lo = thresholds[2 * b], hi = thresholds[2 * b + 1];
        for (int i = tid; i < W; i += ASSIGN_THREADS) {
            float s = scores[w0 + i];   // raw value: NaN compares false both ways -> 4
            int bt = s > hi ? top_bits : (s < lo ? 2 : 4);
            if (pin_first && i == 0) bt = top_bits;
            s_bits[i] = (uint8_t)bt;
        }
    } else {
        int n_top = quota[3 * b], n4 = quota[3 * b + 1];
        int first = 0;
        if (pin_first && W > 0) {
            first = 1;
            if (n_top > 0) n_top--;
            else if (n4 > 0) n4--;
        }
        int n = W - first;
        n_top = min(max(n_top, 0), n);
        n4 = min(max(n4, 0), n - n_top);
        const float4* key4 = reinterpret_cast<const float4*>(s_key);
        for (int i = tid; i < W; i += ASSIGN_THREADS) {
            int bt;
            if (i < first) {
                bt = top_bits;
            } else {
                const float si = s_key[i];
                int r = 0;
                for (int j = 0; j < W4; j += 4) {
                    const float4 k = key4[j >> 2];
                    r += (k.x > si || (k.x == si && j < i)) ? 1 : 0;
                    r += (k.y > si || (k.y == si && j + 1 < i)) ? 1 : 0;
                    r += (k.z > si || (k.z == si && j + 2 < i)) ? 1 : 0;
                    r += (k.w > si || (k.w == si && j + 3 < i)) ? 1 : 0;
                }
                if (first) {            // the pinned window is not part of the ranking
                    const float s0 = s_key[0];
                    r -= (s0 > si || s0 == si) ? 1 : 0;
                }
                bt = r < n_top ? top_bits : (r < n_top + n4 ? 4 : 2);
            }
            s_bits[i] = (uint8_t)bt;
        }
    }
    __syncthreads();
    emit_class_order(s_bits, s_cnt, s_chunk, W, w0, b, bits, perm, seg_windows);
}

// Widths by rank or threshold.  A workgroup takes 64 windows of a sequence; its four wavefronts count, each over a
// quarter of the sequence's keys, how many windows rank before each of the 64 (several workgroups per sequence: a
// sequence of W windows costs W^2 comparisons, which one compute unit alone takes 10 us and more to do from 500 windows on).
constexpr int RANK_THREADS = 256;
constexpr int ASSIGN_ONE_LAUNCH = 320;   // windows per sequence up to which k_assign is taken
__global__ __launch_bounds__(RANK_THREADS) void k_rank(const float* __restrict__ scores, const int32_t* __restrict__ win_off, int mode,
                                                       const int32_t* __restrict__ quota, const float* __restrict__ thresholds,
                                                       int top_bits, int pin_first, uint8_t* __restrict__ bits, int max_windows)
{
    // keys are read four at a time in the counting loop; the array is padded to a multiple of four with -inf, which no
    // key is smaller than and which never counts as an earlier equal
    __shared__ __align__(16) float s_key[WQ_MAX_WINDOWS + 4];
    __shared__ int s_r[RANK_THREADS / 64][64];
    const int b = blockIdx.y;
    const int w0 = win_off[b];
    const int W = min(win_off[b + 1] - w0, max_windows);          // (k_order reports more windows than the caller's bound)
    if ((int)blockIdx.x * 64 >= W) return;
    const int tid = threadIdx.x, lane = tid & 63, part = tid >> 6;
    const int i = (int)blockIdx.x * 64 + lane;
    if (mode == WQ_MODE_THRESHOLD) {
        if (part == 0 && i < W) {
            const float lo = thresholds[2 * b], hi = thresholds[2 * b + 1];
            const float s = scores[w0 + i];      // raw value: NaN compares false both ways -> 4
            int bt = s > hi ? top_bits : (s < lo ? 2 : 4);
            if (pin_first && i == 0) bt = top_bits;
            bits[w0 + i] = (uint8_t)bt;
        }
        return;
    }
    const int W4 = (W + 3) & ~3;
    for (int k = tid; k < W4; k += RANK_THREADS) {
        const float s = k < W ? scores[w0 + k] : -INFINITY;
        s_key[k] = (s != s) ? -INFINITY : s;
    }
    int n_top = quota[3 * b], n4 = quota[3 * b + 1];
    int first = 0;
    if (pin_first && W > 0) {
        first = 1;
        if (n_top > 0) n_top--;
        else if (n4 > 0) n4--;
    }
    const int n = W - first;
    n_top = min(max(n_top, 0), n);
    n4 = min(max(n4, 0), n - n_top);
    __syncthreads();
    // rank_i = #{j : s_j > s_i or (s_j == s_i and j < i)}: this wavefront's quarter of the keys (in fours)
    const int per = (W4 / 4 + RANK_THREADS / 64 - 1) / (RANK_THREADS / 64) * 4;
    const int j0 = part * per, j1 = min(W4, j0 + per);
    const float si = s_key[min(i, W4 - 1)];
    const float4* key4 = reinterpret_cast<const float4*>(s_key);
    int r = 0;
    for (int j = j0; j < j1; j += 4) {
        const float4 k = key4[j >> 2];
        r += (k.x > si || (k.x == si && j < i)) ? 1 : 0;
        r += (k.y > si || (k.y == si && j + 1 < i)) ? 1 : 0;
        r += (k.z > si || (k.z == si && j + 2 < i)) ? 1 : 0;
        r += (k.w > si || (k.w == si && j + 3 < i)) ? 1 : 0;
    }
    s_r[part][lane] = r;
    __syncthreads();
    if (part == 0 && i < W) {
        int bt;
        if (i < first) {
            bt = top_bits;
        } else {
            r = s_r[0][lane] + s_r[1][lane] + s_r[2][lane] + s_r[3][lane];
            static_assert(RANK_THREADS == 256, "four partial counts");
            if (first) {                // the pinned window is not part of the ranking
                const float s0 = s_key[0];
                r -= (s0 > si || s0 == si) ? 1 : 0;
            }
            bt = r < n_top ? top_bits : (r < n_top + n4 ? 4 : 2);
        }
        bits[w0 + i] = (uint8_t)bt;
    }
}

// The class order of widths that are already in `bits`: one workgroup per sequence.
__global__ __launch_bounds__(ASSIGN_THREADS) void k_order(const int32_t* __restrict__ win_off, uint8_t* __restrict__ bits,
                                                          int32_t* __restrict__ perm, int32_t* __restrict__ seg_windows,
                                                          int max_windows, uint32_t* __restrict__ status)
{
    __shared__ __align__(16) uint8_t s_bits[WQ_MAX_WINDOWS + 4];
    __shared__ int s_cnt[4];
    __shared__ int s_chunk[ASSIGN_CHUNKS][4];
    const int b = blockIdx.x;
    const int w0 = win_off[b];
    int W = win_off[b + 1] - w0;
    const int tid = threadIdx.x;
    if (W > max_windows) {                        // more windows than the caller's bound (itself at most WQ_MAX_WINDOWS): reported,
        if (tid == 0) atomicOr(status, WQ_DEV_TOO_MANY_WINDOWS);      // and only the windows inside the bound are assigned
        W = max_windows;
    }
    for (int i = tid; i < W; i += ASSIGN_THREADS) s_bits[i] = bits[w0 + i];
    __syncthreads();
    emit_class_order(s_bits, s_cnt, s_chunk, W, w0, b, bits, perm, seg_windows);
}

// Debug aid: is perm[win_off[b] .. win_off[b+1]) a permutation of 0 .. W_b-1, and do the four class counts of the sequence
// add up to W_b?  One workgroup per sequence, one bit per window in LDS.
__global__ __launch_bounds__(ASSIGN_THREADS) void k_validate(const int32_t* __restrict__ win_off, const int32_t* __restrict__ perm,
                                                             const int32_t* __restrict__ seg_windows, int max_windows,
                                                             uint32_t* __restrict__ status)
{
    __shared__ unsigned s_seen[WQ_MAX_WINDOWS / 32];
    __shared__ int s_bad;
    const int b = blockIdx.x, tid = threadIdx.x;
    const int w0 = win_off[b], W = win_off[b + 1] - w0;
    if (tid == 0) s_bad = 0;
    for (int i = tid; i < WQ_MAX_WINDOWS / 32; i += ASSIGN_THREADS) s_seen[i] = 0u;
    __syncthreads();
    if (W < 0 || W > max_windows) {
        if (tid == 0) atomicOr(status, W < 0 ? WQ_DEV_BAD_ASSIGNMENT : WQ_DEV_TOO_MANY_WINDOWS);
        return;
    }
    for (int i = tid; i < W; i += ASSIGN_THREADS) {
        const int v = perm[w0 + i];
        if (v < 0 || v >= W) s_bad = 1;
        else if (atomicOr(&s_seen[v >> 5], 1u << (v & 31)) & (1u << (v & 31))) s_bad = 1;      // seen before
    }
    if (tid == 0) {
        const int32_t* c = seg_windows + 4 * b;
        if (c[0] < 0 || c[1] < 0 || c[2] < 0 || c[3] < 0 || c[0] + c[1] + c[2] + c[3] != W) s_bad = 1;
    }
    __syncthreads();
    if (tid == 0 && s_bad) atomicOr(status, WQ_DEV_BAD_ASSIGNMENT);
}

}  // namespace

int wq_launch_validate(wq_ctx* ctx, int B, const int32_t* win_off, int max_windows, const int32_t* perm, const int32_t* seg_windows)
{
    hipLaunchKernelGGL(k_validate, dim3(B), dim3(ASSIGN_THREADS), 0, ctx->stream, win_off, perm, seg_windows, max_windows, wq_status_ptr(ctx));
    WQ_HIP_CHECK(ctx, hipGetLastError());
    return WQ_OK;
}

int wq_launch_vote(wq_ctx* ctx, const uint8_t* bits_in, int B, const int32_t* win_off, int max_windows, uint8_t* bits_out, int32_t* perm,
                   int32_t* seg_windows)
{
    hipLaunchKernelGGL(k_vote, dim3(B), dim3(ASSIGN_THREADS), 0, ctx->stream, bits_in, B, win_off, bits_out, perm, seg_windows, max_windows,
                       wq_status_ptr(ctx));
    WQ_HIP_CHECK(ctx, hipGetLastError());
    return WQ_OK;
}

int wq_launch_assign(wq_ctx* ctx, const float* scores, int B, const int32_t* win_off, int max_windows, int mode,
                     const int32_t* quota, const float* thresholds, int top_bits, int pin_first, uint8_t* bits,
                     int32_t* perm, int32_t* seg_windows)
{
    // measured on MI355X: one workgroup per sequence takes 7.9 us + 43 ns per thousand pairs of windows (10.7 us at 256
    // windows, 24.1 at 612), the two launches 13 us whatever the count
    if (max_windows <= ASSIGN_ONE_LAUNCH) {
        hipLaunchKernelGGL(k_assign, dim3(B), dim3(ASSIGN_THREADS), 0, ctx->stream, scores, win_off, mode, quota, thresholds, top_bits,
                           pin_first, bits, perm, seg_windows, max_windows, wq_status_ptr(ctx));
    } else {
        hipLaunchKernelGGL(k_rank, dim3((unsigned)((max_windows + 63) / 64), B), dim3(RANK_THREADS), 0, ctx->stream, scores, win_off, mode,
                           quota, thresholds, top_bits, pin_first, bits, max_windows);
        hipLaunchKernelGGL(k_order, dim3(B), dim3(ASSIGN_THREADS), 0, ctx->stream, win_off, bits, perm, seg_windows, max_windows,
                           wq_status_ptr(ctx));
    }
    WQ_HIP_CHECK(ctx, hipGetLastError());
    return WQ_OK;
}
