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
// c_k = 1/(N |w_k|) sum_j C[k,j] / |t_j|.  A tile is 128 (112, 96) visual rows of one sequence; its text tokens are
// walked in passes of up to 512 columns, so that the visual rows are read from memory once when the sequence has at
// most 512 text tokens.  One workgroup of eight wavefronts per compute unit takes a contiguous share of the launch's
// tiles.  Over D it goes in steps of 128 elements (two 128-byte lines per row):
//   visual rows   memory -> LDS directly (buffer loads with the LDS bit, two steps ahead, three buffers, one barrier per
//                 step) -> A operands of all wavefronts, read two product groups ahead of their use;
//   text rows     each wavefront owns 64 columns of the pass, so its B operands are private to it.  An operand is
//                 16 rows x 16 bytes per lane group: read from the row-major text that is 64 scattered pieces per
//                 load, which the memory pipeline takes one lane at a time.  k_pack_text therefore rewrites the text
//                 once (a few MB) into operand order, [tile of 16 rows][32 elements of D][lane][8 elements], so that
//                 a wavefront's operand is one contiguous KB; it goes from there (L2) straight into registers, a
//                 whole step ahead.
// A wavefront multiplies a [16 RT] x 64 tile per step with v_mfma_f32_16x16x32 bf16/f16 (RT = 8 row tiles: 128
// accumulator registers, two wavefronts per SIMD).  Sequences with at most 256 (128) text tokens use passes of 256
// (128) columns and split the rows between wavefronts instead, RT = 4 (2).  At the end of a pass the products are
// multiplied by 1/|t_j| and summed over the columns, so C never leaves the registers.  |w_k|^2 comes from the A
// operands of one row tile per wavefront during the first pass.  Reductions have a fixed order: results are
// deterministic.
// With operands that change from product to product the matrix cores of this GPU sustain about three quarters of
// their nominal rate (wq_probe_mfma measures it: the clock drops under the load); this kernel keeps them busy three
// quarters of its cycles.  Variants measured and dropped because they were not faster: steps of 64 elements; text
// operands sent for one by one, three quarters of a step ahead; the 32x32x16 form of the instruction.
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
constexpr int PA_PCS = PA_PITCH / 8;     // 16-byte pieces per LDS row, the padding included
constexpr int PA_DMA = (PA_ROWS * PA_PCS + 64 * PA_WAVES - 1) / (64 * PA_WAVES);   // loads to LDS per wavefront and step (64 pieces each)
constexpr int PA_ROW_POLICY = 2;         // cache policy of the visual rows' loads: non-temporal (read once; measured 1 % fewer cycles)
constexpr int PA_BUF = PA_WAVES * PA_DMA * 64 * 8;                                 // elements of one LDS buffer

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

// The three buffers of visual rows are separate arrays on purpose: the compiler then knows that a read of one cannot
// see a load in flight to another, and makes a wavefront wait for exactly the loads it reads behind.
__shared__ __attribute__((aligned(16))) uint16_t pair_a0[PA_BUF];
__shared__ __attribute__((aligned(16))) uint16_t pair_a1[PA_BUF];
__shared__ __attribute__((aligned(16))) uint16_t pair_a2[PA_BUF];
template <int P>
__device__ __forceinline__ uint16_t* pair_buf()
{
    static_assert(P >= 0 && P < 3, "three buffers");
    return P == 0 ? pair_a0 : (P == 1 ? pair_a1 : pair_a2);
}

// x of the lane that a data-parallel-primitive control pairs this lane with (rows of 16 lanes)
template <int CTRL>
__device__ __forceinline__ float pair_lane(float x)
{
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), CTRL, 0xF, 0xF, false));
}

// One stage of a sum over the 16 lanes of a row, for NV values per lane at once: the lane and its partner (which
// differ in `upper`) split the values between them, each adding the other's half of the pair's sums to its own, so
// the lane is left with NV / 2 values, v[0 .. NV/2): the lower half of the indices if !upper, else the upper half.
// With a single value left both keep the sum.
template <int CTRL, int NV>
__device__ __forceinline__ void pair_halve(float (&v)[32], bool upper)
{
    if constexpr (NV >= 2) {
#pragma unroll
        for (int j = 0; j < NV / 2; j++) {
            const float give = upper ? v[j] : v[j + NV / 2];
            const float keep = upper ? v[j + NV / 2] : v[j];
            v[j] = keep + pair_lane<CTRL>(give);
        }
    } else {
        v[0] += pair_lane<CTRL>(v[0]);
    }
}

constexpr int PA_WCAP = 1024;            // text columns whose 1/|t_j| stay in LDS for a whole run
struct PairSmem {
    float W[PA_WCAP];                    // 1/|t_j| (0 past the end): of all passes if they fit, else of the current one
    float R[PA_WAVES][PA_ROWS];          // row sums, one array per column block
    float N2[PA_ROWS];                   // |w_k|^2
};

typedef __attribute__((address_space(3))) void* lds_ptr_t;
template <int P> struct PairBuf { static constexpr int value = P; };
struct PairUnit { int tile, pass; };     // a row tile of the sequence x a pass of columns
struct PairCursor { PairUnit u; int s; }; // a step of a unit

// A run: `ntiles` consecutive row tiles of one sequence, from tile `tile0`, each walked in ceil(N / PASS) passes of PASS
// text columns; a (tile, pass) is a unit of D / 128 steps.  All units of a run form one pipeline: visual rows are sent
// for two steps ahead and text operands one step ahead, across the ends of units, so the matrix cores do not wait for
// memory at the start of a tile, and what a unit leaves behind (scaling by 1/|t_j|, the sum over its columns, at a
// tile's end the scores) happens while those loads are in flight.
// The eight wavefronts are NCB column blocks of 64 text columns x 8 / NCB row groups of RT row tiles of 16:
// (RT, NCB) = (8, 8): 128 rows x a 512-column pass; (4, 4): two row halves x 256 columns; (2, 2): four row quarters
// x 128 columns; (7, 8) and (6, 8): 112 and 96 rows x 512 columns, for launches whose number of 128-row tiles
// would leave most of the chip idle in the last round.  A wavefront whose column block's number is below RT also
// sums |w_k|^2 of the row tile of that number in its row group (read from LDS once more, a quarter at a time).
template <bool BF, int RT, int NCB>
__device__ __forceinline__ void pair_run(PairSmem& sm, const uint16_t* __restrict__ va, const char* __restrict__ tbb,
                                         const float* __restrict__ inv_tn, int D, int M, int N, int tile0, int ntiles, int rows,
                                         float* __restrict__ out)
{
    constexpr int PASS = NCB * PA_WCOLS;                  // columns per pass
    constexpr int DMA = (RT * (PA_WAVES / NCB) * 16 * PA_PCS + 64 * PA_WAVES - 1) / (64 * PA_WAVES);   // loads to LDS per wavefront and step
    static_assert(DMA <= PA_DMA, "LDS buffers too small");
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int lj = lane >> 4, lm = lane & 15;
    const int cb = wave % NCB, rb = (wave / NCB) * RT;
    const int steps = D / PA_KS, ntile = (N + 15) >> 4, npass = (N + PASS - 1) / PASS;

    // visual rows: memory -> LDS without passing registers.  A load instruction fills 64 consecutive 16-byte pieces
    // of the buffer, one per lane; piece p is column p % PA_PCS of row p / PA_PCS.  The descriptor covers the tile's
    // rows only: rows past the sequence's end lie outside it and read as zero, as do the padding columns and the
    // rows past the tile, whose offsets are out of any range.
    auto rows_of = [&](PairUnit u) {
        const int row0 = u.tile * rows;
        return __builtin_amdgcn_make_buffer_rsrc(const_cast<uint16_t*>(va + (int64_t)row0 * D), 0, min(rows, M - row0) * D * 2,
                                                 0x00020000);
    };
    int voff[DMA];
#pragma unroll
    for (int t = 0; t < DMA; t++) {
        const int p = (wave + PA_WAVES * t) * 64 + lane, r = p / PA_PCS, c = p - r * PA_PCS;
        voff[t] = (c < PA_KS / 8 && r < rows) ? (r * D + c * 8) * 2 : (int)0x80000000;
    }
    auto send_rows = [&](auto P, __amdgpu_buffer_rsrc_t tile_rows, int byte0) {     // 256 bytes of every row, from byte0 -> buffer P
        uint16_t* const dst = pair_buf<decltype(P)::value>();
#pragma unroll
        for (int t = 0; t < DMA; t++)
            __builtin_amdgcn_raw_ptr_buffer_load_lds(tile_rows, (lds_ptr_t)(dst + (wave + PA_WAVES * t) * 512), 16, voff[t], byte0, 0,
                                                     PA_ROW_POLICY);
    };
    // byte offset of this lane's operand piece in a row tile's first quarter: of the wavefront's first tile (the
    // tiles follow each other by 16 rows), and of the tile whose |w_k|^2 it sums
    constexpr int TILE_BYTES = 16 * PA_PITCH * 2;
    const int ro = ((rb * 16 + lm) * PA_PITCH + lj * 8) * 2, ro_own = ro + (cb < RT ? cb : 0) * TILE_BYTES;
    // A read from the buffer that this wavefront has sent loads for: the compiler puts the wait for those loads in
    // front of it (loads land in the order sent), whatever else it has moved around them.
    auto peek = [&](auto P) {
        const char* const src = reinterpret_cast<const char*>(pair_buf<decltype(P)::value>());
        return *reinterpret_cast<const uint32_t*>(src + ro);
    };
    auto use = [&](uint32_t x) { asm volatile("" ::"v"(x)); };
    // the wavefront's column tiles of a pass in the packed text (tiles past the end re-read the last one: their
    // weights are zero); a lane's 16 bytes of operand c of a tile sit at 1024 c + 16 lane
    auto text_of = [&](PairUnit u, const char* (&t)[PA_CT]) {
#pragma unroll
        for (int k = 0; k < PA_CT; k++)
            t[k] = tbb + (int64_t)min((u.pass * PASS + cb * PA_WCOLS) / 16 + k, ntile - 1) * (D / 32) * 1024;
    };
    auto load_b = [&](const char* const (&t)[PA_CT], int c, uint4 (&gb)[PA_CT]) {      // elements 32 c .. 32 c + 31 of D
        const uint32_t off = (uint32_t)(c * 1024) + (uint32_t)lane * 16u;
#pragma unroll
        for (int k = 0; k < PA_CT; k++) gb[k] = *reinterpret_cast<const uint4*>(t[k] + off);
    };
    auto after = [&](PairUnit u) {                        // the unit after u; the run's last unit is followed by itself
        if (++u.pass == npass) { u.pass = 0; ++u.tile; }
        if (u.tile == tile0 + ntiles) { u.tile = tile0 + ntiles - 1; u.pass = npass - 1; }
        return u;
    };
    // 1/|t_j| in LDS: all passes' at once if they fit, else pass by pass (the slow way: behind a barrier at a unit's end)
    const bool w_all = npass * PASS <= PA_WCAP;
    auto stage_weights = [&](int col0, int n) {
        for (int k = threadIdx.x; k < n; k += PA_THREADS) sm.W[k] = col0 + k < N ? inv_tn[col0 + k] : 0.f;
    };

    // Three cursors walk the run's steps: (uc, s) the step whose products are being summed; cb_, one step ahead, the
    // step whose text operands are sent for (tc: its unit's text); ca, two steps ahead, the step whose visual rows are
    // sent for (dc: its tile's rows).  Past the run's end they stay in its last unit.
    auto advance = [&](PairCursor& c) {                   // true when it has entered another unit
        if (++c.s < steps) return false;
        c.s = 0;
        c.u = after(c.u);
        return true;
    };
    PairUnit uc{tile0, 0};
    PairCursor cb_{uc, 0}, ca{uc, 0};
    __amdgpu_buffer_rsrc_t dc = rows_of(uc);
    const char* tc[PA_CT];
    text_of(uc, tc);
    floatx4s acc[RT][PA_CT];
#pragma unroll
    for (int i = 0; i < RT; i++)
#pragma unroll
        for (int k = 0; k < PA_CT; k++) acc[i][k] = floatx4s{0.f, 0.f, 0.f, 0.f};
    float nsq = 0.f;
    int s = 0;

    __syncthreads();                                      // whoever used the buffers before is done with them
    stage_weights(0, w_all ? npass * PASS : PASS);
    __syncthreads();
    // gq[q]: B operands of quarter q of a step, sent for a whole step ahead (replaced one by one during the following
    // quarter, three quarters ahead, they cost 8 % more cycles: the text does not always come from the nearest cache)
    uint4 gq[PA_Q][PA_CT];
    send_rows(PairBuf<0>{}, dc, 0);
    if (advance(ca)) dc = rows_of(ca.u);
    send_rows(PairBuf<1>{}, dc, ca.s * (PA_KS * 2));
    if (advance(ca)) dc = rows_of(ca.u);
#pragma unroll
    for (int q = 0; q < PA_Q; q++) load_b(tc, q, gq[q]);
    if (advance(cb_)) text_of(cb_.u, tc);
    use(peek(PairBuf<0>{}));

    // What a unit leaves behind.  The lane holds, of its i-th row tile, rows 4 lj + e at column lm of column tile k.
    // Scale by 1/|t_j| and sum over the wavefront's 64 columns: over k in the lane, over lm across the 16 lanes of a
    // row in four stages of pairwise exchanges, each of which halves the number of values a lane carries (the
    // partners are lm ^ 8, lm ^ 7, lm ^ 2, lm ^ 1; the stages split on bits 3, 2, 1, 0 of lm).
    // (Both work from a copy of the thread's number that the compiler cannot trace: what they derive from it is then
    // computed here, once per unit, rather than kept in registers throughout the steps.)
    auto unit_done = [&]() {
        int t = tid;
        asm volatile("" : "+v"(t));
        const int lm = t & 15, lj = (t >> 4) & 3;
        float wk[PA_CT];
#pragma unroll
        for (int k = 0; k < PA_CT; k++) wk[k] = sm.W[(w_all ? uc.pass * PASS : 0) + cb * PA_WCOLS + k * 16 + lm];
        float v[32];
#pragma unroll
        for (int i = 0; i < RT; i++)
#pragma unroll
            for (int e = 0; e < 4; e++) {
                float x = 0.f;
#pragma unroll
                for (int k = 0; k < PA_CT; k++) x = fmaf(acc[i][k][e], wk[k], x);
                v[i * 4 + e] = x;
            }
#pragma unroll
        for (int i = 0; i < RT; i++)
#pragma unroll
            for (int k = 0; k < PA_CT; k++) acc[i][k] = floatx4s{0.f, 0.f, 0.f, 0.f};
        constexpr int NV = RT > 4 ? 32 : RT * 4;            // a power of two
#pragma unroll
        for (int j = RT * 4; j < NV; j++) v[j] = 0.f;
        pair_halve<0x128, NV>(v, (lm & 8) != 0);                    // row_ror:8
        pair_halve<0x141, NV / 2>(v, (lm & 4) != 0);                // row_half_mirror
        pair_halve<0x4E, (NV >= 4 ? NV / 4 : 1)>(v, (lm & 2) != 0); // quad_perm [2,3,0,1]
        pair_halve<0xB1, (NV >= 8 ? NV / 8 : 1)>(v, (lm & 1) != 0); // quad_perm [1,0,3,2]
        // what is left: values j0 .. j0 + KEEP - 1 of the NV (j = 4 i + e), j0 made of the bits of lm that split a
        // stage; a stage that did not split left the sum in both lanes, the lower one writes
        constexpr int KEEP = NV >= 16 ? NV / 16 : 1;
        int j0 = 0;
        bool writer = true;
        if constexpr (NV >= 2) j0 += (lm & 8) ? NV / 2 : 0;
        if constexpr (NV >= 4) j0 += (lm & 4) ? NV / 4 : 0;
        if constexpr (NV >= 8) j0 += (lm & 2) ? NV / 8 : 0; else writer = writer && !(lm & 2);
        if constexpr (NV >= 16) j0 += (lm & 1) ? NV / 16 : 0; else writer = writer && !(lm & 1);
        if (writer) {
#pragma unroll
            for (int r = 0; r < KEEP; r++) {
                const int j = j0 + r, tile = rb + (j >> 2);
                if ((j >> 2) < RT) sm.R[cb][tile * 16 + 4 * lj + (j & 3)] += v[r];    // one writer per (column block, row)
            }
        }
    };
    // A tile's last unit is done: its scores.  |w_k|^2: a wavefront summed row tile number `wave` (in every tiling the
    // first tile it walks; with seven or six tiles the last wavefronts summed nothing and write zeros to rows that do
    // not exist); its lane (lm, lj) holds the sum over the pieces lj, lj + 4, ... of row lm.
    auto tile_done = [&](int tile) {
        int tid = threadIdx.x;
        asm volatile("" : "+v"(tid));
        const int lane = tid & 63;
        nsq += __shfl_xor(nsq, 16, 64);
        nsq += __shfl_xor(nsq, 32, 64);
        if (lane < 16) sm.N2[wave * 16 + lane] = nsq;
        nsq = 0.f;
        asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");      // (no fence: loads for the next unit are in flight)
        const int row = tile * rows + tid;
        if (tid < PA_ROWS) {
            float r = 0.f;
#pragma unroll
            for (int c = 0; c < PA_WAVES; c++) {
                r += sm.R[c][tid];
                sm.R[c][tid] = 0.f;                       // for the next tile; the barriers of its steps come before its sums
            }
            const float nn = sm.N2[tid];
            if (tid < rows && row < M) out[row] = nn > 0.f ? r / (sqrtf(nn) * (float)N) : 0.f;
        }
    };

    // A step: LDS buffer P x the B operands, a quarter (32 elements of D) at a time.  The products' part has no
    // branches: it stays one block, which keeps the wait counts of the loads in flight exact.
    auto step = [&](auto P) {
        using Cur = decltype(P);
        using Nxt = PairBuf<(Cur::value + 1) % 3>;
        using Far = PairBuf<(Cur::value + 2) % 3>;
        // every wavefront's rows of this step have landed (each waited for its own before it came here), and all are
        // done reading the buffer of the step before, which takes the rows two steps ahead.  No fence: a fence would
        // wait for the B operands in flight.
        asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
        __builtin_amdgcn_sched_barrier(0);
        send_rows(Far{}, dc, ca.s * (PA_KS * 2));
        const float count = (uc.pass == 0 && cb < RT) ? 1.f : 0.f;   // |w_k|^2 is summed during the first pass, by the tile's owner (a factor, not a branch)
        const char* const sa = reinterpret_cast<const char*>(pair_buf<Cur::value>());
        // PA_Q RT groups of PA_CT products: row tile i, quarter q; the A operand is read from LDS two groups
        // ahead.  A quarter's B operands are replaced as soon as their last product has issued.
        auto read_a = [&](int g) { return *reinterpret_cast<const uint4*>(sa + ro + (g % RT) * TILE_BYTES + (g / RT) * 64); };
        uint4 f[3], own;
        uint32_t landed = 0u;
        f[0] = read_a(0);
        f[1] = read_a(1);
#pragma unroll
        for (int g = 0; g < PA_Q * RT; g++) {
            const int i = g % RT, q = g / RT;
            if (g + 2 < PA_Q * RT) f[(g + 2) % 3] = read_a(g + 2);
            if (i == 0) own = *reinterpret_cast<const uint4*>(sa + ro_own + q * 64);
            if (g == PA_Q * RT - 2) landed = peek(Nxt{});             // waits for the next step's rows, as late as it can
            if (i == RT - 1) nsq = fmaf(sumsq8<BF>(own), count, nsq);
#pragma unroll
            for (int k = 0; k < PA_CT; k++) acc[i][k] = mfma_s<BF>(f[g % 3], gq[q][k], acc[i][k]);
            if (i == RT - 1) load_b(tc, PA_Q * cb_.s + q, gq[q]);
            __builtin_amdgcn_sched_barrier(0);            // issue order as written: one LDS read, then the group's products
        }
        use(landed);
        if (s == steps - 1) {
            const PairUnit un = after(uc);
            unit_done();
            if (uc.pass == npass - 1) tile_done(uc.tile);
            if (!w_all) {
                asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");      // all have read this unit's weights
                stage_weights(un.pass * PASS, PASS);
            }
            s = 0;
            uc = un;
        } else {
            ++s;
        }
        if (advance(cb_)) text_of(cb_.u, tc);
        if (advance(ca)) dc = rows_of(ca.u);
    };
    const int total = ntiles * npass * steps;
    int gs = 0;
    for (; gs + 2 < total; gs += 3) {
        step(PairBuf<0>{});
        step(PairBuf<1>{});
        step(PairBuf<2>{});
    }
    if (gs < total) step(PairBuf<0>{});
    if (gs + 1 < total) step(PairBuf<1>{});
    use(peek(PairBuf<0>{}));                              // nothing of this run is in flight to LDS any more
    use(peek(PairBuf<1>{}));
    use(peek(PairBuf<2>{}));
}

// The launch's row tiles (`rows` = 128, 112 or 96 visual rows) are numbered sequence after sequence; a workgroup takes
// a contiguous share of them and walks it as runs of tiles of one sequence.
template <bool BF>
__global__ __launch_bounds__(PA_THREADS) __attribute__((amdgpu_waves_per_eu(2, 2))) void k_pair_mfma(const uint16_t* __restrict__ vis, const uint4* __restrict__ packed_txt,
                                                          const float* __restrict__ inv_tnorm, int D, int B,
                                                          const int32_t* __restrict__ vis_off, const int32_t* __restrict__ txt_off,
                                                          int rows, float* __restrict__ tok_score)
{
    __shared__ PairSmem sm;
    const int tid = threadIdx.x;
    uint32_t T = 0;
    for (int b = 0; b < B; b++) T += (uint32_t)(vis_off[b + 1] - vis_off[b] + rows - 1) / (uint32_t)rows;
    int g = (int)((uint64_t)T * blockIdx.x / gridDim.x);
    const int end = (int)((uint64_t)T * (blockIdx.x + 1) / gridDim.x);
    if (g >= end) return;
    for (int k = tid; k < PA_WAVES * PA_ROWS; k += PA_THREADS) sm.R[k / PA_ROWS][k % PA_ROWS] = 0.f;     // (a run starts with a barrier)
    int b = 0, first = 0;                                 // first: number of sequence b's first tile
    while (g < end) {
        int Tb = (vis_off[b + 1] - vis_off[b] + rows - 1) / rows;
        while (g >= first + Tb) {
            first += Tb;
            ++b;
            Tb = (vis_off[b + 1] - vis_off[b] + rows - 1) / rows;
        }
        const int n = min(end, first + Tb) - g, tile0 = g - first;
        const int m0 = vis_off[b], M = vis_off[b + 1] - m0;
        const int n0 = txt_off[b], N = txt_off[b + 1] - n0;
        const uint16_t* va = vis + (int64_t)m0 * D;
        const char* tb = reinterpret_cast<const char*>(packed_txt) + (int64_t)pair_tile_base(txt_off, b) * (D / 32) * 1024;
        float* out = tok_score + m0;
        if (N <= 0) {
            for (int r = tile0 * rows + tid; r < min(M, (tile0 + n) * rows); r += PA_THREADS) out[r] = 0.f;
        } else if (N > 4 * PA_WCOLS) {
            if (rows == 128)
                pair_run<BF, 8, 8>(sm, va, tb, inv_tnorm + n0, D, M, N, tile0, n, rows, out);
            else if (rows == 112)
                pair_run<BF, 7, 8>(sm, va, tb, inv_tnorm + n0, D, M, N, tile0, n, rows, out);
            else
                pair_run<BF, 6, 8>(sm, va, tb, inv_tnorm + n0, D, M, N, tile0, n, rows, out);
        } else if (N > 2 * PA_WCOLS) {                    // (fewer rows than 128: the last row tiles are empty)
            pair_run<BF, 4, 4>(sm, va, tb, inv_tnorm + n0, D, M, N, tile0, n, rows, out);
        } else {
            pair_run<BF, 2, 2>(sm, va, tb, inv_tnorm + n0, D, M, N, tile0, n, rows, out);
        }
        g += n;
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
            // rows per workgroup: a workgroup occupies a compute unit, so the launch runs in rounds of as many
            // workgroups as the chip has compute units; take the size whose rounds cover the fewest rows in all
            static int cus = 0;
            if (cus <= 0) {
                int dev = 0;
                if (hipGetDevice(&dev) != hipSuccess ||
                    hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus <= 0)
                    cus = 256;
            }
            int rows = PA_ROWS;
            int64_t best = 0;
            for (int r = PA_ROWS; r >= 96; r -= 16) {
                const int64_t wgs = (total_vis + r - 1) / r, cost = ((wgs + cus - 1) / cus) * r;
                if (r == PA_ROWS || cost < best) { best = cost; rows = r; }
            }
            // one workgroup per compute unit, or fewer if there are fewer tiles (a sequence has at most one partial tile)
            const int64_t tiles_most = (total_vis + rows - 1) / rows + B;
            const dim3 grid((unsigned)(tiles_most < cus ? tiles_most : cus));
            if (dtype == WQ_BF16)
                hipLaunchKernelGGL(k_pair_mfma<true>, grid, dim3(PA_THREADS), 0, st, v16, packed, inv_norm, D, B, vis_off, txt_off, rows, tok_score);
            else
                hipLaunchKernelGGL(k_pair_mfma<false>, grid, dim3(PA_THREADS), 0, st, v16, packed, inv_norm, D, B, vis_off, txt_off, rows, tok_score);
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
