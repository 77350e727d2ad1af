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

#include <type_traits>

namespace {

constexpr int WAVE = 64;
// k_token_score: visual rows per wavefront, and how far the loop over a row's elements is unrolled (measured on 4 x 50176 rows of
// 3584 bf16: 2 rows, unrolled twice: 257 us for the whole call; 4 rows: 277; 1 row: 269; 8 rows: 390)
constexpr int WQ_TS_ROWS = 2;
#define WQ_TS_UNROLL 2

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

// tbar[b][d] = 1/N sum_j t_j[d]/|t_j|.  VEC: a workgroup takes 64 columns, thread = (8 columns, one of 32 token slices),
// slices merged in LDS in slice order (many small workgroups: the kernel is bound by the latency of its row loads);
// otherwise one thread per column.
template <typename T, bool VEC>
__global__ __launch_bounds__(256) void k_text_mean(const T* __restrict__ txt, const float* __restrict__ inv_norm, int D,
                                                   const int32_t* __restrict__ txt_off, float* __restrict__ tbar)
{
    const int b = blockIdx.y;
    const int j0 = txt_off[b], j1 = txt_off[b + 1];
    if (VEC) {
        __shared__ float s_acc[32][8][9];
        const int cc = threadIdx.x & 7, ts = threadIdx.x >> 3;
        const int d0 = (blockIdx.x * 8 + cc) * 8;
        float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
        if (d0 < D)
            for (int j = j0 + ts; j < j1; j += 32) {
                float x[8];
                wq_ld8(txt + (int64_t)j * D + d0, x);
                const float w = inv_norm[j];
#pragma unroll
                for (int k = 0; k < 8; k++) acc[k] = fmaf(x[k], w, acc[k]);
            }
#pragma unroll
        for (int k = 0; k < 8; k++) s_acc[ts][cc][k] = acc[k];
        __syncthreads();
        const int c2 = threadIdx.x >> 3, k2 = threadIdx.x & 7;      // 8 chunks x 8 columns
        const int d = (blockIdx.x * 8 + c2) * 8 + k2;
        if (threadIdx.x < 64 && d < D) {
            float s = 0.f;
#pragma unroll
            for (int t = 0; t < 32; t++) s += s_acc[t][c2][k2];
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

// c_k = (w_k . tbar) / |w_k|.  VEC: one wavefront takes WQ_TS_ROWS consecutive rows so that each 32-byte piece of the pooled
// text vector is loaded once per WQ_TS_ROWS rows; 16 bytes of every row per lane and iteration.
template <typename T, bool VEC>
__global__ __launch_bounds__(256) void k_token_score(const T* __restrict__ vis, const float* __restrict__ tbar, int D, int B,
                                                     const int32_t* __restrict__ vis_off, int64_t total_vis,
                                                     float* __restrict__ tok_score)
{
    const int lane = threadIdx.x & 63;
    if (VEC) {
        constexpr int R = WQ_TS_ROWS;
        const int64_t row0 = ((int64_t)blockIdx.x * 4 + (threadIdx.x >> 6)) * R;
        if (row0 >= total_vis) return;
        int bs[R];
        const T* p[R];
#pragma unroll
        for (int r = 0; r < R; r++) {
            const int64_t row = row0 + r < total_vis ? row0 + r : total_vis - 1;
            bs[r] = wq_find_seq(vis_off, B, row);
            p[r] = vis + row * D;
        }
        const bool same = bs[0] == bs[R - 1];      // rows are ordered by sequence: all of them share one text vector
        float ss[R], dt[R];
#pragma unroll
        for (int r = 0; r < R; r++) ss[r] = dt[r] = 0.f;
#pragma unroll WQ_TS_UNROLL
        for (int d = lane * 8; d < D; d += WAVE * 8) {
            float t[8];
            wq_ld8(tbar + (int64_t)bs[0] * D + d, t);
#pragma unroll
            for (int r = 0; r < R; r++) {
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
        for (int r = 0; r < R; r++) {
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
// c_k = 1/(N |w_k|) sum_j C[k,j] / |t_j|.  One workgroup of eight wavefronts owns 128 visual rows of one sequence and
// walks the text tokens in passes of up to 512 columns, so that the visual rows are read from memory once when the
// sequence has at most 512 text tokens.  Over D it goes in steps of 128 elements (two 128-byte lines per row):
//   visual rows   global -> registers (a step ahead) -> LDS (two buffers, one barrier per step) -> A operands of
//                 all wavefronts, read two products groups ahead of their use;
//   text rows     each wavefront owns 64 columns of the pass, so its B operands are private to it.  An operand is
//                 16 rows x 16 bytes per lane group: read from the row-major text that is 64 scattered pieces per
//                 load, which the memory pipeline takes one lane at a time.  k_pack_text therefore rewrites the text
//                 once (a few MB) into operand order, [tile of 16 rows][32 elements of D][lane][8 elements], so that
//                 a wavefront's operand is one contiguous KB; it goes from there (L2) straight into registers, a
//                 quarter of a step ahead.
// A wavefront multiplies a [16 RT] x 64 tile per step with v_mfma_f32_16x16x32 bf16/f16 (RT = 8 row tiles: 128
// accumulator registers, two wavefronts per SIMD).  Sequences with at most 256 (128) text tokens use passes of 256
// (128) columns and split the rows between wavefronts instead, RT = 4 (2).  The epilogue of a pass multiplies by
// 1/|t_j| and reduces over the columns, so C never leaves the registers.  |w_k|^2 comes from the visual rows on
// their way to LDS during the first pass.  Reductions have a fixed order: results are deterministic.
// With operands that change from product to product the matrix cores of this GPU sustain about two thirds of their
// nominal rate (wq_probe_mfma measures it: the clock drops under the load); this kernel reaches somewhat more than
// half of that.  Variants measured and dropped because they were not faster: visual rows sent straight into LDS
// (no registers) with B operands three quarters of a step ahead; steps of 64 elements.
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

typedef __bf16 bf16x2s __attribute__((ext_vector_type(2)));
typedef _Float16 half2s __attribute__((ext_vector_type(2)));

// sum of the squares of eight 16-bit elements (v_dot2_f32: both products and the sum in fp32)
template <bool BF>
__device__ __forceinline__ float sumsq8(const uint4& u)
{
    const uint32_t w[4] = {u.x, u.y, u.z, u.w};
    float s = 0.f;
#pragma unroll
    for (int k = 0; k < 4; k++) {
        if constexpr (BF) {
            const bf16x2s p = __builtin_bit_cast(bf16x2s, w[k]);
            s = __builtin_amdgcn_fdot2_f32_bf16(p, p, s, false);
        } else {
            const half2s p = __builtin_bit_cast(half2s, w[k]);
            s = __builtin_amdgcn_fdot2(p, p, s, false);
        }
    }
    return s;
}

constexpr int PA_THREADS = 512, PA_WAVES = 8;
constexpr int PA_ROWS = 128;             // visual rows per workgroup
constexpr int PA_KS = 128;               // elements of D per step (two 128-byte lines per row)
constexpr int PA_Q = PA_KS / 32;         // quarters of a step: one matrix instruction deep each
constexpr int PA_PITCH = PA_KS + 16;     // LDS row pitch in elements (288 bytes: rows start 32 bytes apart in the banks; measured free of bank conflicts, a pitch of 272 bytes is not)
constexpr int PA_WCOLS = 64;             // text columns per wavefront and pass
constexpr int PA_CT = PA_WCOLS / 16;     // column tiles per wavefront
constexpr int PA_PPR = PA_KS / 8;        // 16-byte pieces per row and step
constexpr int PA_RPT = PA_THREADS / PA_PPR;   // rows that the workgroup stages at a time
constexpr int PA_NU = PA_ROWS / PA_RPT;  // pieces per thread and step

// Tiles of 16 text rows in operand order.  Sequence b's tiles start at tile txt_off[b] / 16 + b: room for
// ceil(N_b / 16) tiles each, whatever the lengths.  Rows past N_b are zero.
__device__ __forceinline__ int pair_tile_base(const int32_t* txt_off, int b) { return (txt_off[b] >> 4) + b; }

__global__ __launch_bounds__(256) void k_pack_text(const uint16_t* __restrict__ txt, int D, int B, const int32_t* __restrict__ txt_off,
                                                   int64_t total_tiles, uint4* __restrict__ packed)
{
    const int chunks = D / 32;
    const int64_t item = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);      // (tile, chunk of 32 elements)
    if (item >= total_tiles * chunks) return;
    const int64_t tile = item / chunks;
    const int c = (int)(item - tile * chunks), lane = threadIdx.x & 63, lm = lane & 15, lj = lane >> 4;
    // the sequence that owns this tile: the last b with pair_tile_base(b) <= tile
    int lo = 0, hi = B - 1;
    while (lo < hi) {
        const int mid = (lo + hi + 1) >> 1;
        if (pair_tile_base(txt_off, mid) <= tile) lo = mid; else hi = mid - 1;
    }
    const int n0 = txt_off[lo], N = txt_off[lo + 1] - n0;
    const int row = (int)(tile - pair_tile_base(txt_off, lo)) * 16 + lm;
    uint4 v = make_uint4(0u, 0u, 0u, 0u);
    if (row < N) v = *reinterpret_cast<const uint4*>(txt + ((int64_t)n0 + row) * D + c * 32 + lj * 8);
    packed[item * 64 + lane] = v;
}

struct PairSmem {
    __attribute__((aligned(16))) uint16_t A[2][PA_ROWS * PA_PITCH];
    float W[PA_WAVES * PA_WCOLS];        // 1/|t_j| of the pass (0 past the end)
    float R[PA_WAVES][PA_ROWS];          // row sums, one array per column block
    float N2[PA_ROWS];                   // |w_k|^2
};

// RT row tiles of 16 per wavefront: 8 -> the eight wavefronts are eight column blocks of a 512-column pass,
// 4 -> two row halves x four column blocks (256 columns), 2 -> four row quarters x two column blocks (128).
template <bool BF, int RT>
__device__ __forceinline__ void pair_body(PairSmem& sm, const uint16_t* __restrict__ va, const char* __restrict__ tbb,
                                          const float* __restrict__ inv_tn, int D, int M, int N, int row0, float (&nsq)[PA_NU])
{
    constexpr int NCB = RT, PASS = NCB * PA_WCOLS;        // column blocks per pass
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int lj = lane >> 4, lm = lane & 15;
    const int cb = wave % NCB, rb = (wave / NCB) * RT;
    const int pp = tid % PA_PPR, pr = tid / PA_PPR;       // visual rows to LDS: thread -> 16-byte piece pp of rows pr + PA_RPT u
    const uint16_t* pa[PA_NU];
#pragma unroll
    for (int u = 0; u < PA_NU; u++) pa[u] = va + (int64_t)min(row0 + pr + PA_RPT * u, M - 1) * D + pp * 8;   // rows past the end re-read the last
    const int steps = D / PA_KS, ntile = (N + 15) >> 4;

    auto load_a = [&](int s, uint4 (&ga)[PA_NU]) {
#pragma unroll
        for (int u = 0; u < PA_NU; u++) ga[u] = *reinterpret_cast<const uint4*>(pa[u] + s * PA_KS);
    };
    // count: 1 when these rows have not been summed into |w_k|^2 yet, else 0 (a factor, not a branch: the loop body
    // stays one block, which keeps the wait counts of the loads in flight exact)
    auto store_a = [&](int buf, const uint4 (&ga)[PA_NU], float count) {
#pragma unroll
        for (int u = 0; u < PA_NU; u++) {
            *reinterpret_cast<uint4*>(&sm.A[0][(pr + PA_RPT * u) * PA_PITCH + pp * 8] + buf * (PA_ROWS * PA_PITCH)) = ga[u];
            nsq[u] = fmaf(sumsq8<BF>(ga[u]), count, nsq[u]);
        }
    };

    for (int c0 = 0; c0 < N; c0 += PASS) {
        const bool first_pass = c0 == 0;
        // this wavefront's column tiles in the packed text: byte offsets (32 bits: checked by the host) of the lane's
        // 16 bytes in the tile's first operand; tiles past the end re-read the last one (their weights are zero)
        uint32_t ob[PA_CT];
#pragma unroll
        for (int k = 0; k < PA_CT; k++)
            ob[k] = (uint32_t)min((c0 + cb * PA_WCOLS) / 16 + k, ntile - 1) * (uint32_t)(D / 32) * 1024u + (uint32_t)lane * 16u;
        auto load_b = [&](int c, uint4 (&gb)[PA_CT]) {    // elements 32 c .. 32 c + 31 of D
#pragma unroll
            for (int k = 0; k < PA_CT; k++) gb[k] = *reinterpret_cast<const uint4*>(tbb + (ob[k] + (uint32_t)(c * 1024)));
        };
        floatx4s acc[RT][PA_CT];
#pragma unroll
        for (int i = 0; i < RT; i++)
#pragma unroll
            for (int k = 0; k < PA_CT; k++) acc[i][k] = floatx4s{0.f, 0.f, 0.f, 0.f};

        __syncthreads();                                  // the previous pass is done with W and with both A buffers
        for (int k = tid; k < PASS; k += PA_THREADS) sm.W[k] = (c0 + k < N) ? inv_tn[c0 + k] : 0.f;
        // gx, gy: B operands of the even and odd quarters of a step; ga: visual rows of the next step
        uint4 ga[PA_NU], gx[PA_CT], gy[PA_CT];
        const int last_c = D / 32 - 1;
        load_b(0, gx);
        load_b(1, gy);
        load_a(0, ga);
        store_a(0, ga, first_pass ? 1.f : 0.f);
        load_a(min(1, steps - 1), ga);

        // step s: LDS buffer s % 2 x the B operands, a quarter (32 elements of D) at a time.  No branches: the body
        // stays one block, which keeps the wait counts of the loads in flight exact.  Past the end the last
        // operands are fetched again, unused.
        for (int s = 0; s < steps; s++) {
            const int buf = s & 1;
            __syncthreads();                              // A tile of step s is written; the other buffer is free
            __builtin_amdgcn_sched_barrier(0);
            const uint16_t* sa = &sm.A[0][(rb * 16 + lm) * PA_PITCH + lj * 8] + buf * (PA_ROWS * PA_PITCH);
            // PA_Q RT groups of PA_CT products: row tile i, quarter q; the A operand is read from LDS two groups
            // ahead.  A quarter's B operands are replaced as soon as their last product has issued, so they have
            // a quarter of a step to arrive (the packed text is in L2).
            auto read_a = [&](int g) { return *reinterpret_cast<const uint4*>(sa + (g % RT) * 16 * PA_PITCH + (g / RT) * 32); };
            uint4 f[3];
            f[0] = read_a(0);
            f[1] = read_a(1);
#pragma unroll
            for (int g = 0; g < PA_Q * RT; g++) {
                const int i = g % RT, q = g / RT;
                if (g + 2 < PA_Q * RT) f[(g + 2) % 3] = read_a(g + 2);
#pragma unroll
                for (int k = 0; k < PA_CT; k++) acc[i][k] = mfma_s<BF>(f[g % 3], (q & 1) == 0 ? gx[k] : gy[k], acc[i][k]);
                if (i == RT - 1) {                        // quarter q is done: its buffer takes quarter q + 2
                    const int c = min(PA_Q * s + q + 2, last_c);
                    if ((q & 1) == 0) load_b(c, gx); else load_b(c, gy);
                }
                __builtin_amdgcn_sched_barrier(0);        // issue order as written: one LDS read, then the group's products
            }
            // the next step's rows (sent for a step ago) go to the other LDS buffer; then send for the rows after them
            store_a(buf ^ 1, ga, (first_pass && s + 1 < steps) ? 1.f : 0.f);
            load_a(min(s + 2, steps - 1), ga);
        }

        // epilogue: lane holds rows 4 lj + e of row tile i, column lm of column tile k
        float wk[PA_CT];
#pragma unroll
        for (int k = 0; k < PA_CT; k++) wk[k] = sm.W[cb * PA_WCOLS + k * 16 + lm];
#pragma unroll
        for (int i = 0; i < RT; i++) {
#pragma unroll
            for (int e = 0; e < 4; e++) {
                float v = 0.f;
#pragma unroll
                for (int k = 0; k < PA_CT; k++) v = fmaf(acc[i][k][e], wk[k], v);
                v += __shfl_xor(v, 1, 64);
                v += __shfl_xor(v, 2, 64);
                v += __shfl_xor(v, 4, 64);
                v += __shfl_xor(v, 8, 64);
                if (lm == 0) sm.R[cb][(rb + i) * 16 + 4 * lj + e] += v;     // one writer per (column block, row)
            }
        }
    }
}

template <bool BF>
__global__ __launch_bounds__(PA_THREADS) __attribute__((amdgpu_waves_per_eu(2, 2))) void k_pair_mfma(const uint16_t* __restrict__ vis, const uint4* __restrict__ packed_txt,
                                                          const float* __restrict__ inv_tnorm, int D,
                                                          const int32_t* __restrict__ vis_off, const int32_t* __restrict__ txt_off,
                                                          float* __restrict__ tok_score)
{
    __shared__ PairSmem sm;
    const int b = blockIdx.y;
    const int m0 = vis_off[b], M = vis_off[b + 1] - m0;
    const int n0 = txt_off[b], N = txt_off[b + 1] - n0;
    const int row0 = blockIdx.x * PA_ROWS;
    if (row0 >= M) return;
    const int tid = threadIdx.x;
    for (int k = tid; k < PA_WAVES * PA_ROWS; k += PA_THREADS) sm.R[k / PA_ROWS][k % PA_ROWS] = 0.f;
    float nsq[PA_NU];
#pragma unroll
    for (int u = 0; u < PA_NU; u++) nsq[u] = 0.f;
    const uint16_t* va = vis + (int64_t)m0 * D;
    const char* tb = reinterpret_cast<const char*>(packed_txt) + (int64_t)pair_tile_base(txt_off, b) * (D / 32) * 1024;
    if (N > 4 * PA_WCOLS)
        pair_body<BF, 8>(sm, va, tb, inv_tnorm + n0, D, M, N, row0, nsq);
    else if (N > 2 * PA_WCOLS)
        pair_body<BF, 4>(sm, va, tb, inv_tnorm + n0, D, M, N, row0, nsq);
    else
        pair_body<BF, 2>(sm, va, tb, inv_tnorm + n0, D, M, N, row0, nsq);
    // |w_k|^2: the PA_PPR threads that staged a row hold its 16-byte pieces of every step
    const int pp = tid % PA_PPR, pr = tid / PA_PPR;
#pragma unroll
    for (int u = 0; u < PA_NU; u++) {
        float v = nsq[u];
#pragma unroll
        for (int o = 1; o < PA_PPR; o <<= 1) v += __shfl_xor(v, o, 64);
        if (pp == 0) sm.N2[pr + PA_RPT * u] = v;
    }
    __syncthreads();
    if (tid < PA_ROWS && row0 + tid < M) {
        float r = 0.f;
#pragma unroll
        for (int c = 0; c < PA_WAVES; c++) r += sm.R[c][tid];
        const float nn = sm.N2[tid];
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
    hipLaunchKernelGGL((k_text_mean<T, VEC>), dim3(VEC ? (D + 63) / 64 : (D + 255) / 256, B), dim3(256), 0, st, txt, inv_norm, D, txt_off, tbar);
    if (total_vis > 0) {
        const int64_t rows_per_block = VEC ? 4 * WQ_TS_ROWS : 4;
        hipLaunchKernelGGL((k_token_score<T, VEC>), dim3((unsigned)((total_vis + rows_per_block - 1) / rows_per_block)), dim3(256), 0, st,
                           vis, tbar, D, B, vis_off, total_vis, tok_score);
    }
    hipLaunchKernelGGL(k_window_mean, dim3((unsigned)((total_win + 3) / 4)), dim3(256), 0, st, tok_score, B, vis_off, txt_off,
                       win_size, win_off, total_win, scores);
    WQ_HIP_CHECK(ctx, hipGetLastError());
    return WQ_OK;
}

}  // namespace

// tiles of 16 text rows that the packed text of B sequences with total_txt rows can take (see pair_tile_base)
static int64_t pair_total_tiles(int B, int64_t total_txt) { return total_txt / 16 + B; }

size_t wq_scores_ws_bytes(int B, int64_t total_vis, int64_t total_txt, int D)
{
    if (B <= 0 || D <= 0) return 0;
    return wq_align256(sizeof(float) * (size_t)(total_txt > 0 ? total_txt : 1)) + wq_align256(sizeof(float) * (size_t)B * D) +
           wq_align256(sizeof(float) * (size_t)(total_vis > 0 ? total_vis : 1)) +
           wq_align256((size_t)pair_total_tiles(B, total_txt) * 16 * (size_t)D * 2);      // text in operand order (pairwise path)
}

int wq_launch_scores(wq_ctx* ctx, const void* vis, const void* txt, int dtype, int B, int D, const int32_t* vis_off,
                     const int32_t* txt_off, const int32_t* win_size, const int32_t* win_off, int64_t total_vis,
                     int64_t total_txt, int64_t total_win, int algo, float* scores)
{
    if (algo == WQ_SCORE_PAIRWISE_MFMA) {
        if (D % 128 != 0) return wq_fail(ctx, WQ_ERR_UNSUPPORTED, "the matrix-core scoring path needs D %% 128 == 0");
        if ((reinterpret_cast<uintptr_t>(vis) | reinterpret_cast<uintptr_t>(txt)) % 16 != 0)
            return wq_fail(ctx, WQ_ERR_ARG, "embeddings must be 16-byte aligned");
        const int64_t tiles = pair_total_tiles(B, total_txt);
        if (tiles * 16 * (int64_t)D * 2 > (int64_t)UINT32_MAX)
            return wq_fail(ctx, WQ_ERR_UNSUPPORTED, "the matrix-core scoring path takes at most 4 GiB of text embeddings");
        char* ws = ctx->ws + WQ_WS_HEADER;
        float* inv_norm = reinterpret_cast<float*>(ws);
        ws += wq_align256(sizeof(float) * (size_t)(total_txt > 0 ? total_txt : 1));
        ws += wq_align256(sizeof(float) * (size_t)B * D);
        float* tok_score = reinterpret_cast<float*>(ws);
        ws += wq_align256(sizeof(float) * (size_t)(total_vis > 0 ? total_vis : 1));
        uint4* packed = reinterpret_cast<uint4*>(ws);
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
            const int64_t items = tiles * (D / 32);
            hipLaunchKernelGGL(k_pack_text, dim3((unsigned)((items + 3) / 4)), dim3(256), 0, st, t16, D, B, txt_off, tiles, packed);
            // any one sequence has at most total_vis rows: row tiles past a sequence's end return at once
            const dim3 grid((unsigned)((total_vis + PA_ROWS - 1) / PA_ROWS), B);
            if (dtype == WQ_BF16)
                hipLaunchKernelGGL(k_pair_mfma<true>, grid, dim3(PA_THREADS), 0, st, v16, packed, inv_norm, D, vis_off, txt_off, tok_score);
            else
                hipLaunchKernelGGL(k_pair_mfma<false>, grid, dim3(PA_THREADS), 0, st, v16, packed, inv_norm, D, vis_off, txt_off, tok_score);
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
