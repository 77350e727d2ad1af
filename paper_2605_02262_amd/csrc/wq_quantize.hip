// a3: reorder + asymmetric round-to-nearest quantization + packing (Sec. 3.3.1, Sec. 3.3.3, Alg. 2 prefill half).
//
//   k_plan      one workgroup: per-class padded offsets / lengths of every sequence, 16-bit row counts,
//               capacity checks (device status word)
//   k_quantize_all  one launch for the three classes and the 16-bit rows.  A class workgroup takes one
//               (32-token destination block, KV head): gathers the source rows through
//               perm (the window reorder is fused into the load), finds each group's min/max with
//               wavefront shuffles, computes codes with the exact fp32 sequence of the format definition,
//               stages them in LDS and writes the K tile / V block / metadata images with coalesced stores
//               The remaining workgroups copy one row each of the 16-bit windows, video tail and text -> k16/v16
// HBM-bound: reads 2 x 2 bytes per (K,V) element pair once, writes b/8 + 4/group bytes per element.
// This file is compiled with floating-point contraction off: the code sequence must round exactly as stated.
#include <type_traits>

#include "wq_internal.h"

#pragma clang fp contract(off)

namespace {

__device__ __forceinline__ int pad32(int n) { return (n + 31) & ~31; }

__global__ __launch_bounds__(256) void k_plan(int B, const int32_t* __restrict__ kv_off, const int32_t* __restrict__ win_size,
                                              const int32_t* __restrict__ win_off, const int32_t* __restrict__ seg_windows,
                                              wq_packed_kv pk, int32_t* __restrict__ pre16, uint32_t* __restrict__ status)
{
    const int tid = threadIdx.x;
    if (tid < 3) {
        const int c = tid;
        int32_t* off = pk.cls_off[c];
        int32_t* len = pk.cls_len[c];
        int64_t run = 0;
        bool over = false;
        off[0] = 0;
        for (int b = 0; b < B; b++) {
            int n = seg_windows[4 * b + c] * win_size[b];
            int64_t nxt = run + pad32(n);
            if (nxt > pk.cap[c]) {          // does not fit: drop the sequence's share of this class
                over = true;
                n = 0;
                nxt = run;
            }
            len[b] = n;
            run = nxt;
            off[b + 1] = (int32_t)run;
        }
        if (over) atomicOr(status, WQ_DEV_CLASS_OVERFLOW);
    } else if (tid == 3) {
        int64_t run = 0;
        bool over = false;
        pre16[0] = 0;
        for (int b = 0; b < B; b++) {
            int W = win_off[b + 1] - win_off[b];
            int rows = kv_off[b + 1] - kv_off[b];
            int n = seg_windows[4 * b + 3] * win_size[b] + (rows - W * win_size[b]);
            int room = pk.off16[b + 1] - pk.off16[b];
            if (n > room || (int64_t)pk.off16[b] + n > pk.cap16 || pk.off16[b] < 0) {
                over = true;
                n = 0;
            }
            pk.len16[b] = n;
            run += n;
            pre16[b + 1] = (int32_t)run;
        }
        if (over) atomicOr(status, WQ_DEV_SEG16_OVERFLOW);
    } else if (tid >= 64) {
        for (int b = tid - 64; b < B; b += 192) pk.v_scale_max[b] = 0.f;      // k_v_scale_max raises it
    }
}

// maximum of a small unsigned value over the 64 lanes of a wavefront: four rotations inside the rows of 16 lanes (one
// data-parallel-primitive instruction each, no LDS), then the four rows' results as scalars
template <int CTRL>
__device__ __forceinline__ uint32_t lanes_moved(uint32_t x)
{
    return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, CTRL, 0xF, 0xF, false);
}
__device__ __forceinline__ uint32_t lanes_max_u16(uint32_t x)
{
    x = max(x, lanes_moved<0x128>(x));             // row_ror:8, 4, 2, 1
    x = max(x, lanes_moved<0x124>(x));
    x = max(x, lanes_moved<0x122>(x));
    x = max(x, lanes_moved<0x121>(x));
    const uint32_t a = (uint32_t)__builtin_amdgcn_readlane((int)x, 0), b = (uint32_t)__builtin_amdgcn_readlane((int)x, 16);
    const uint32_t c = (uint32_t)__builtin_amdgcn_readlane((int)x, 32), d = (uint32_t)__builtin_amdgcn_readlane((int)x, 48);
    return max(max(a, b), max(c, d));
}

// v_scale_max holds [B] results, then one float per (32-token block, KV head) of the three classes (class c's blocks
// behind those of the classes before it, by capacity)
__device__ __forceinline__ int64_t v_scale_slot(const wq_packed_kv& pk, int B, int c, int64_t blk, int kvh)
{
    int64_t base = 0;
    for (int k = 0; k < c; k++) base += pk.cap[k] / 32;
    return (int64_t)B + (base + blk) * pk.Hkv + kvh;
}

// per sequence: the largest of its blocks' largest value scales (0 if it has no quantized token).  WQ_VS_PARTS workgroups
// per sequence take a slice of the blocks each and raise the sequence's entry, which k_plan has set to zero (positive
// floats order like their bit patterns)
constexpr int WQ_VS_PARTS = 16;
__global__ __launch_bounds__(256) void k_v_scale_max(int B, wq_packed_kv pk)
{
    __shared__ float red[256];
    const int b = blockIdx.x / WQ_VS_PARTS, part = blockIdx.x % WQ_VS_PARTS, tid = threadIdx.x;
    float mx = 0.f;
    for (int c = 0; c < 3; c++) {
        const int64_t t0 = pk.cls_off[c][b] / 32, t1 = pk.cls_off[c][b + 1] / 32;
        const int64_t first = v_scale_slot(pk, B, c, t0, 0), n = (t1 - t0) * pk.Hkv;
        const int64_t per = (n + WQ_VS_PARTS - 1) / WQ_VS_PARTS, lo = part * per, hi = min(n, lo + per);
        const float* src = pk.v_scale_max + first;
        int64_t i = lo + tid;
        for (; i + 768 < hi; i += 1024) {          // four loads in flight
            const float a0 = src[i], a1 = src[i + 256], a2 = src[i + 512], a3 = src[i + 768];
            mx = fmaxf(fmaxf(mx, a0), fmaxf(fmaxf(a1, a2), a3));
        }
        for (; i < hi; i += 256) mx = fmaxf(mx, src[i]);
    }
    red[tid] = mx;
    __syncthreads();
    for (int o = 128; o >= 1; o >>= 1) {
        if (tid < o) red[tid] = fmaxf(red[tid], red[tid + o]);
        __syncthreads();
    }
    if (tid == 0 && red[0] > 0.f) atomicMax(reinterpret_cast<unsigned*>(pk.v_scale_max + b), __float_as_uint(red[0]));
}

// bits -> class index
__host__ __device__ constexpr int cls_index(int bits) { return bits == 2 ? 0 : (bits == 4 ? 1 : 2); }

// V codes of a 32-token block on their way into operand order, one byte each: the 8 tokens x HD/16 channel tiles of a
// lane of the decode kernel's matrix operand (lane = 16 jj + mm holds channels 16 ct + mm of tokens 16 (tau >> 2) +
// 4 jj + (tau & 3)) lie together, [ct][tau], at lane x VT_PITCH; the 16 bytes of padding keep the readers' 16-byte
// reads in different banks
template <int HD>
struct QuantSmem {
    static constexpr int VT_PITCH = (HD / 16) * 8 + 16;
    __attribute__((aligned(16))) uint8_t vt[64 * VT_PITCH];
    uint32_t meta[2][4][32];                    // [plane][group][token]
};

template <int CTRL>
__device__ __forceinline__ float lanes_moved_f(float x)
{
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), CTRL, 0xF, 0xF, false));
}

// 16 codes of BITS bits, one per byte of x[0..3], as consecutive fields: 2 BITS bytes in y
template <int BITS>
__device__ __forceinline__ void pack16(const uint32_t (&x)[4], uint32_t (&y)[4])
{
    if constexpr (BITS == 8) {
#pragma unroll
        for (int i = 0; i < 4; i++) y[i] = x[i];
    } else if constexpr (BITS == 4) {
#pragma unroll
        for (int i = 0; i < 2; i++) {
            const uint32_t a = x[2 * i] | (x[2 * i] >> 4), b = x[2 * i + 1] | (x[2 * i + 1] >> 4);     // bytes 0 and 2 hold two codes each
            y[i] = __builtin_amdgcn_perm(b, a, 0x06040200u);                                          // a.b0 a.b2 b.b0 b.b2
        }
    } else {
        uint32_t z[4];
#pragma unroll
        for (int i = 0; i < 4; i++) {
            const uint32_t a = x[i] | (x[i] >> 6);          // bytes 0 and 2 hold two codes each
            z[i] = a | (a >> 12);                           // byte 0 holds all four
        }
        y[0] = __builtin_amdgcn_perm(__builtin_amdgcn_perm(z[3], z[2], 0x0C0C0400u), __builtin_amdgcn_perm(z[1], z[0], 0x0C0C0400u), 0x05040100u);
    }
}

// one (32-token destination block `blk` of class BITS, KV head `kvh`)
template <typename T, int HD, int BITS>
__device__ __forceinline__ void quantize_block(QuantSmem<HD>& sm, int blk, int kvh, const T* __restrict__ K, const T* __restrict__ V,
                                               int B, int group, const int32_t* __restrict__ kv_off,
                                               const int32_t* __restrict__ win_size, const int32_t* __restrict__ win_off,
                                               const int32_t* __restrict__ perm, const int32_t* __restrict__ seg_windows,
                                               const wq_packed_kv& pk, uint32_t* __restrict__ status)
{
    constexpr int C = cls_index(BITS);
    constexpr int QMAX = (1 << BITS) - 1;
    constexpr int CPT = HD / 8;                 // channels per thread: 8 threads share one token row
    constexpr int PER_DW = 32 / BITS;           // codes per output dword
    auto& s_meta = sm.meta;
    const int tid = threadIdx.x;
    const int Hkv = pk.Hkv;
    const int G = HD / group;
    const int32_t* off = pk.cls_off[C];
    const int64_t tok0 = (int64_t)blk * 32;
    if (tok0 >= off[B]) return;                 // unused capacity
    const int b = wq_find_seq(off, B, tok0);
    const int d0 = (int)(tok0 - off[b]);        // first destination token of the block inside the segment
    const int len = pk.cls_len[C][b];
    const int S = win_size[b];
    int pos0 = 0;                               // windows of lower classes come first in perm
    for (int c = 0; c < C; c++) pos0 += seg_windows[4 * b + c];

    // ---- gather + quantize: thread = (token u, part p) -------------------------------------------------
    const int u = tid >> 3, p = tid & 7;
    const int d = d0 + u;
    const bool valid = d < len;
    int64_t src = 0;
    if (valid) {
        int r = d / S, o = d - r * S;
        int win = perm[win_off[b] + pos0 + r];
        src = (int64_t)kv_off[b] + (int64_t)win * S + o;
    }
    const int tpg = group / CPT;                // threads per group (2, 4 or 8; 16 when group=128, hd=64 is excluded)
#pragma unroll
    for (int plane = 0; plane < 2; plane++) {
        const T* X = plane == 0 ? K : V;
        float x[CPT];
        float lo = INFINITY, hi = -INFINITY;
        if (valid) {
            const int64_t base = (src * Hkv + kvh) * HD + p * CPT;
#pragma unroll
            for (int i = 0; i < CPT; i += 8) wq_ld8(X + base + i, x + i);     // 16-byte pieces (rows are 16-byte aligned)
#pragma unroll
            for (int i = 0; i < CPT; i++) {
                lo = fminf(lo, x[i]);
                hi = fmaxf(hi, x[i]);
            }
        } else {
#pragma unroll
            for (int i = 0; i < CPT; i++) x[i] = 0.f;
            lo = hi = 0.f;
        }
        // lanes p..p+tpg-1 of a token are adjacent lanes of one wavefront: partners p ^ 1, p ^ 2, p ^ 7 (lane moves
        // inside quads and half rows, no LDS)
        lo = fminf(lo, lanes_moved_f<0xB1>(lo));
        hi = fmaxf(hi, lanes_moved_f<0xB1>(hi));
        if (tpg >= 4) {
            lo = fminf(lo, lanes_moved_f<0x4E>(lo));
            hi = fmaxf(hi, lanes_moved_f<0x4E>(hi));
        }
        if (tpg >= 8) {
            lo = fminf(lo, lanes_moved_f<0x141>(lo));
            hi = fmaxf(hi, lanes_moved_f<0x141>(hi));
        }
        if (lo == 0.0f) lo = 0.0f;               // a zero minimum is stored as +0
        const __half mh = __float2half_rn(lo);
        const float m = __half2float(mh);
        const float r = hi - m;
        const float s0 = r / (float)QMAX;       // correctly rounded fp32 divide
        __half sh = __float2half_rn(s0);
        float s = __half2float(sh);
        if (s == 0.0f) {
            s = 1.0f;
            sh = __float2half_rn(1.0f);
        }
        const float inv = 1.0f / s;
        // This thread's codes: the K plane takes them as consecutive BITS-wide fields of its token's row quarter
        // (pw, stored below); the V plane goes through LDS, a byte per code, to where the operand order wants it.
        // A token past the end has x = 0 everywhere, which gives m = 0, s = 1 and codes 0.
        constexpr int NB = CPT * BITS / 8;      // bytes of the K fields: 2..16
        uint32_t pw[(NB + 3) / 4];
#pragma unroll
        for (int i = 0; i < (NB + 3) / 4; i++) pw[i] = 0;
        uint8_t* const vt = sm.vt + ((u >> 2) & 3) * (16 * QuantSmem<HD>::VT_PITCH) + (u & 3) + 4 * (u >> 4);    // lane 16 jj (+ mm), byte tau (+ 8 ct)
#pragma unroll
        for (int i = 0; i < CPT; i++) {
            float t = (x[i] - m) * inv;         // contraction is off: subtract, round, multiply, round
            float q = rintf(t);
            q = __builtin_amdgcn_fmed3f(q, 0.0f, (float)QMAX);      // (the clamp: no NaN comes here)
            const uint32_t code = (uint32_t)(int)q;
            if (plane == 0) {
                pw[(i * BITS) >> 5] |= code << ((i * BITS) & 31);
            } else {
                const int ch = p * CPT + i;     // (ch & 15, ch >> 4 are fixed per i once p is known: CPT divides 16)
                vt[(ch & 15) * QuantSmem<HD>::VT_PITCH + (ch >> 4) * 8] = (uint8_t)code;
            }
        }
        if (plane == 0) {
            constexpr int Q = HD / 4;
            const int j = (p * CPT) / Q, e0 = (p * CPT) % Q;
            uint8_t* out = static_cast<uint8_t*>(pk.codes[C]) + ((int64_t)kvh * pk.cap[C] + tok0) * HD * BITS / 8 +
                           (u >> 4) * (16 * HD * BITS / 8) + ((j * 16 + (u & 15)) * Q + e0) * BITS / 8;
            if constexpr (NB == 2) {
                *reinterpret_cast<uint16_t*>(out) = (uint16_t)pw[0];
            } else if constexpr (NB == 4) {
                *reinterpret_cast<uint32_t*>(out) = pw[0];
            } else if constexpr (NB == 8) {
                *reinterpret_cast<uint2*>(out) = uint2{pw[0], pw[1]};
            } else {
                *reinterpret_cast<uint4*>(out) = uint4{pw[0], pw[1], pw[2], pw[3]};
            }
        }
        if ((p * CPT) % group == 0) {
            uint32_t word = valid ? ((uint32_t)__half_as_ushort(sh) | ((uint32_t)__half_as_ushort(mh) << 16)) : 0u;
            s_meta[plane][(p * CPT) / group][u] = word;
        }
    }
    __syncthreads();

    // ---- the block's largest value scale (the decode kernel places its fp16 weights by the sequence's largest one): the
    //      scales are the low halves of the V metadata words, zero for tokens past the end; positive f16 values order like
    //      their bit patterns.  One plain store per workgroup into the table's scratch part; k_v_scale_max collects them ----
    if (tid < 64) {
        uint32_t top = 0;
        for (int i = tid; i < 32 * G; i += 64) top = max(top, s_meta[1][i >> 5][i & 31] & 0xFFFFu);
        top = lanes_max_u16(top);
        if (tid == 0) pk.v_scale_max[v_scale_slot(pk, B, C, blk, kvh)] = wq_f16_bits_to_float(top);
    }

    // ---- V plane: block of 32 tokens, field n = ((jj*16 + mm)*(HD/16) + ct)*8 + tau: LDS holds the codes in this
    //      order, a byte each; a thread packs 16 of them (two channel tiles of a lane) into 2 BITS bytes ----------
    {
        constexpr int CT = HD / 16;
        uint8_t* out = static_cast<uint8_t*>(pk.codes[C]) + (((int64_t)Hkv + kvh) * pk.cap[C] + tok0) * HD * BITS / 8;
        for (int r = tid; r < 64 * CT / 2; r += 256) {
            const uint4 c = *reinterpret_cast<const uint4*>(sm.vt + (r / (CT / 2)) * QuantSmem<HD>::VT_PITCH + (r % (CT / 2)) * 16);
            const uint32_t x[4] = {c.x, c.y, c.z, c.w};
            uint32_t y[4];
            pack16<BITS>(x, y);
            if constexpr (BITS == 8)
                *reinterpret_cast<uint4*>(out + r * 16) = uint4{y[0], y[1], y[2], y[3]};
            else if constexpr (BITS == 4)
                *reinterpret_cast<uint2*>(out + r * 8) = uint2{y[0], y[1]};
            else
                *reinterpret_cast<uint32_t*>(out + r * 4) = y[0];
        }
    }
    // ---- metadata: [tile of 16][group][16 tokens] ---------------------------------------------------------
    {
        const int lg = G >> 1;                  // log2 of G = 1, 2 or 4: at most 256 words, one per thread
        if (tid < (64 << lg)) {
            const int plane = tid >> (5 + lg), r = tid & ((32 << lg) - 1);
            const int tile = r >> (4 + lg), gi = (r >> 4) & (G - 1), mrow = r & 15;
            uint32_t* out = static_cast<uint32_t*>(pk.meta[C]) + (((int64_t)plane * Hkv + kvh) * pk.cap[C] + tok0) * G;
            out[r] = s_meta[plane][gi][tile * 16 + mrow];
        }
    }
}

// row r of all 16-bit rows of the batch
template <typename T>
__device__ __forceinline__ void copy16_row(int64_t r, const T* __restrict__ K, const T* __restrict__ V, int B, int row_elems,
                                           const int32_t* __restrict__ kv_off, const int32_t* __restrict__ win_size,
                                           const int32_t* __restrict__ win_off, const int32_t* __restrict__ perm,
                                           const int32_t* __restrict__ seg_windows, const int32_t* __restrict__ pre16,
                                           const wq_packed_kv& pk)
{
    if (r >= pre16[B]) return;
    const int b = wq_find_seq(pre16, B, r);
    const int i = (int)(r - pre16[b]);
    const int S = win_size[b];
    const int W = win_off[b + 1] - win_off[b];
    const int n16w = seg_windows[4 * b + 3] * S;
    int64_t src;
    if (i < n16w) {
        int pos0 = seg_windows[4 * b] + seg_windows[4 * b + 1] + seg_windows[4 * b + 2];
        int rr = i / S, o = i - rr * S;
        src = (int64_t)kv_off[b] + (int64_t)perm[win_off[b] + pos0 + rr] * S + o;
    } else {
        src = (int64_t)kv_off[b] + (int64_t)W * S + (i - n16w);
    }
    const int64_t dst = (int64_t)pk.off16[b] + i;
    uint16_t* k16 = static_cast<uint16_t*>(pk.k16) + dst * row_elems;
    uint16_t* v16 = static_cast<uint16_t*>(pk.v16) + dst * row_elems;
    for (int e = threadIdx.x; e < row_elems; e += 256) {
        float kx = wq_ld(K, src * row_elems + e), vx = wq_ld(V, src * row_elems + e);
        if constexpr (std::is_same_v<T, __hip_bfloat16>) {          // bf16 -> bf16
            k16[e] = (uint16_t)(__float_as_uint(kx) >> 16);
            v16[e] = (uint16_t)(__float_as_uint(vx) >> 16);
        } else {                                                           // fp16 / fp32 -> fp16 (nearest even)
            k16[e] = __half_as_ushort(__float2half_rn(kx));
            v16[e] = __half_as_ushort(__float2half_rn(vx));
        }
    }
}

// The whole call after k_plan in one launch: workgroups [0, n0) take the 2-bit blocks, [n0, n1) the 4-bit blocks,
// [n1, n2) the 8-bit blocks (consecutive workgroups = the KV heads of one token block: together they read whole source
// rows), the rest one 16-bit row each.
template <typename T, int HD>
__global__ __launch_bounds__(256) void k_quantize_all(const T* __restrict__ K, const T* __restrict__ V, int B, int group,
                                                      const int32_t* __restrict__ kv_off, const int32_t* __restrict__ win_size,
                                                      const int32_t* __restrict__ win_off, const int32_t* __restrict__ perm,
                                                      const int32_t* __restrict__ seg_windows, const int32_t* __restrict__ pre16,
                                                      wq_packed_kv pk, unsigned n0, unsigned n1, unsigned n2, uint32_t* __restrict__ status)
{
    __shared__ QuantSmem<HD> sm;
    const unsigned w = blockIdx.x;
    const unsigned Hkv = (unsigned)pk.Hkv;
    if (w < n0)
        quantize_block<T, HD, 2>(sm, (int)(w / Hkv), (int)(w % Hkv), K, V, B, group, kv_off, win_size, win_off, perm, seg_windows, pk, status);
    else if (w < n1)
        quantize_block<T, HD, 4>(sm, (int)((w - n0) / Hkv), (int)((w - n0) % Hkv), K, V, B, group, kv_off, win_size, win_off, perm, seg_windows, pk, status);
    else if (w < n2)
        quantize_block<T, HD, 8>(sm, (int)((w - n1) / Hkv), (int)((w - n1) % Hkv), K, V, B, group, kv_off, win_size, win_off, perm, seg_windows, pk, status);
    else
        copy16_row<T>((int64_t)(w - n2), K, V, B, pk.Hkv * HD, kv_off, win_size, win_off, perm, seg_windows, pre16, pk);
}

// one generated token per sequence -> the end of its 16-bit segment
template <typename T>
__global__ __launch_bounds__(256) void k_append16(const T* __restrict__ k_new, const T* __restrict__ v_new, int row_elems,
                                                  wq_packed_kv pk, uint32_t* __restrict__ status)
{
    const int b = blockIdx.x;
    const int64_t row = (int64_t)pk.off16[b] + pk.len16[b];
    const bool full = row >= pk.off16[b + 1] || row >= pk.cap16;
    __syncthreads();                       // every lane has read len16[b] before it changes
    if (full) {
        if (threadIdx.x == 0) atomicOr(status, WQ_DEV_SEG16_OVERFLOW);
        return;
    }
    uint16_t* k16 = static_cast<uint16_t*>(pk.k16) + row * row_elems;
    uint16_t* v16 = static_cast<uint16_t*>(pk.v16) + row * row_elems;
    for (int e = threadIdx.x; e < row_elems; e += 256) {
        const float kx = wq_ld(k_new, (int64_t)b * row_elems + e), vx = wq_ld(v_new, (int64_t)b * row_elems + e);
        if constexpr (std::is_same_v<T, __hip_bfloat16>) {
            k16[e] = (uint16_t)(__float_as_uint(kx) >> 16);
            v16[e] = (uint16_t)(__float_as_uint(vx) >> 16);
        } else {
            k16[e] = __half_as_ushort(__float2half_rn(kx));
            v16[e] = __half_as_ushort(__float2half_rn(vx));
        }
    }
    if (threadIdx.x == 0) pk.len16[b] += 1;
}

// ---- the unfused variant of the operator-fusion ablation (Sec. 3.3.3, Sec. 4.4): packed classes back to 16-bit rows -------------
// dst's 16-bit segment receives, per sequence, the dequantized tokens of src's 2-, 4- and 8-bit classes (in this order,
// the order of the cache) and then src's 16-bit rows; dst's classes are empty.  Decode attention over dst is then the
// plain 16-bit attention that a dequantize-to-memory implementation would run.
//   k_dense_plan   dst tables, capacity check
//   k_dequantize   one workgroup per (32-token block of a class, KV head): value = fma(code, s, m) in fp32, rounded to
//                  nearest even into the 16-bit type
//   k_dense_copy   src's 16-bit rows
__device__ __forceinline__ int dense_total(const wq_packed_kv& src, int b)
{
    return src.cls_len[0][b] + src.cls_len[1][b] + src.cls_len[2][b] + src.len16[b];
}
__device__ __forceinline__ bool dense_fits(const wq_packed_kv& src, const wq_packed_kv& dst, int b)
{
    const int n = dense_total(src, b);
    return dst.off16[b] >= 0 && n <= dst.off16[b + 1] - dst.off16[b] && (int64_t)dst.off16[b] + n <= dst.cap16;
}

__global__ __launch_bounds__(256) void k_dense_plan(int B, wq_packed_kv src, wq_packed_kv dst, uint32_t* __restrict__ status)
{
    for (int b = threadIdx.x; b < B; b += 256) {
        const bool ok = dense_fits(src, dst, b);
        dst.len16[b] = ok ? dense_total(src, b) : 0;
        if (!ok) atomicOr(status, WQ_DEV_SEG16_OVERFLOW);
#pragma unroll
        for (int c = 0; c < 3; c++) dst.cls_len[c][b] = 0;
        dst.v_scale_max[b] = 0.f;
    }
    for (int b = threadIdx.x; b <= B; b += 256)
#pragma unroll
        for (int c = 0; c < 3; c++) dst.cls_off[c][b] = 0;
}

__device__ __forceinline__ uint16_t to_16bit(float x, bool bf16)
{
    if (bf16) {
        const uint32_t u = __float_as_uint(x);
        return (uint16_t)((u + 0x7FFFu + ((u >> 16) & 1u)) >> 16);       // nearest even (finite values)
    }
    return __half_as_ushort(__float2half_rn(x));
}

template <int HD, int BITS>
__global__ __launch_bounds__(256) void k_dequantize(int B, wq_packed_kv src, wq_packed_kv dst)
{
    constexpr int C = cls_index(BITS);
    constexpr int CPT = HD / 8;                 // channels per thread: 8 threads share one token row
    constexpr int Q = HD / 4, CT = HD / 16;
    constexpr int BLK_B = 32 * HD * BITS / 8;   // bytes of a 32-token block of one plane
    __shared__ __align__(16) uint8_t s_v[BLK_B];
    const int tid = threadIdx.x, kvh = blockIdx.y, Hkv = src.Hkv, G = HD / src.group;
    const int32_t* off = src.cls_off[C];
    const int64_t tok0 = (int64_t)blockIdx.x * 32;
    if (tok0 >= off[B]) return;                 // unused capacity
    const int b = wq_find_seq(off, B, tok0);
    if (!dense_fits(src, dst, b)) return;
    const int d0 = (int)(tok0 - off[b]), len = src.cls_len[C][b];
    int before = 0;                             // tokens of the lower classes come first
    for (int c = 0; c < C; c++) before += src.cls_len[c][b];
    const bool bf16 = dst.dtype16 == WQ_BF16;

    const uint8_t* kc = static_cast<const uint8_t*>(src.codes[C]) + ((int64_t)kvh * src.cap[C] + tok0) * HD * BITS / 8;
    const uint8_t* vc = static_cast<const uint8_t*>(src.codes[C]) + (((int64_t)Hkv + kvh) * src.cap[C] + tok0) * HD * BITS / 8;
    for (int i = tid; i < BLK_B / 16; i += 256) reinterpret_cast<uint4*>(s_v)[i] = reinterpret_cast<const uint4*>(vc)[i];
    __syncthreads();

    const int u = tid >> 3, p = tid & 7;        // token of the block, part of its row
    if (d0 + u >= len) return;
    const int64_t row = (int64_t)dst.off16[b] + before + d0 + u;
    const int tile = u >> 4, m = u & 15;
    const int gi = (p * CPT) / src.group;       // the thread's channels lie in one group (group >= CPT)
    uint32_t ko[CPT / 2], vo[CPT / 2];              // pairs of 16-bit values
#pragma unroll
    for (int i = 0; i < CPT / 2; i++) ko[i] = vo[i] = 0u;
    {   // K: the thread's codes are consecutive fields of its token's row quarter
        const uint32_t word = static_cast<const uint32_t*>(src.meta[C])[((int64_t)kvh * src.cap[C] + tok0) * G + (tile * G + gi) * 16 + m];
        const float s = __half2float(__ushort_as_half((uint16_t)(word & 0xFFFFu))), mn = __half2float(__ushort_as_half((uint16_t)(word >> 16)));
        const int j = (p * CPT) / Q, e0 = (p * CPT) % Q;
        const uint8_t* in = kc + tile * (16 * HD * BITS / 8) + ((j * 16 + m) * Q + e0) * BITS / 8;
        constexpr int NB = CPT * BITS / 8;      // bytes of the thread's codes: 2..16, aligned to their size
        uint32_t pw[(NB + 3) / 4];
        if constexpr (NB == 2) {
            pw[0] = *reinterpret_cast<const uint16_t*>(in);
        } else if constexpr (NB == 4) {
            pw[0] = *reinterpret_cast<const uint32_t*>(in);
        } else if constexpr (NB == 8) {
            const uint2 t = *reinterpret_cast<const uint2*>(in);
            pw[0] = t.x, pw[1] = t.y;
        } else {
            const uint4 t = *reinterpret_cast<const uint4*>(in);
            pw[0] = t.x, pw[1] = t.y, pw[2] = t.z, pw[3] = t.w;
        }
#pragma unroll
        for (int i = 0; i < CPT; i++) {
            const uint32_t code = (pw[(i * BITS) >> 5] >> ((i * BITS) & 31)) & ((1u << BITS) - 1u);
            ko[i >> 1] |= (uint32_t)to_16bit(fmaf((float)code, s, mn), bf16) << (16 * (i & 1));
        }
    }
    {   // V: field n = ((jj*16 + mm)*CT + ct)*8 + tau of the block, channel 16 ct + mm
        const uint32_t word = static_cast<const uint32_t*>(src.meta[C])[(((int64_t)Hkv + kvh) * src.cap[C] + tok0) * G + (tile * G + gi) * 16 + m];
        const float s = __half2float(__ushort_as_half((uint16_t)(word & 0xFFFFu))), mn = __half2float(__ushort_as_half((uint16_t)(word >> 16)));
        const int jj = m >> 2, tau = 4 * tile + (u & 3);
#pragma unroll
        for (int i = 0; i < CPT; i++) {
            const int ch = p * CPT + i, ct = ch >> 4, mm = ch & 15;
            const int bit = (((jj * 16 + mm) * CT + ct) * 8 + tau) * BITS;
            const uint32_t code = (s_v[bit >> 3] >> (bit & 7)) & ((1u << BITS) - 1u);
            vo[i >> 1] |= (uint32_t)to_16bit(fmaf((float)code, s, mn), bf16) << (16 * (i & 1));
        }
    }
    uint16_t* k16 = static_cast<uint16_t*>(dst.k16) + (row * Hkv + kvh) * HD + p * CPT;
    uint16_t* v16 = static_cast<uint16_t*>(dst.v16) + (row * Hkv + kvh) * HD + p * CPT;
#pragma unroll
    for (int i = 0; i < CPT; i += 8) {
        *reinterpret_cast<uint4*>(k16 + i) = make_uint4(ko[i / 2], ko[i / 2 + 1], ko[i / 2 + 2], ko[i / 2 + 3]);
        *reinterpret_cast<uint4*>(v16 + i) = make_uint4(vo[i / 2], vo[i / 2 + 1], vo[i / 2 + 2], vo[i / 2 + 3]);
    }
}

__global__ __launch_bounds__(256) void k_dense_copy(int B, int row_elems, wq_packed_kv src, wq_packed_kv dst)
{
    const int64_t r = blockIdx.x;               // a row of src's 16-bit segment
    const int b = wq_find_seq(src.off16, B, r);
    if (r < src.off16[0] || r >= src.off16[B]) return;
    const int i = (int)(r - src.off16[b]);
    if (i >= src.len16[b] || !dense_fits(src, dst, b)) return;
    const int64_t d = (int64_t)dst.off16[b] + src.cls_len[0][b] + src.cls_len[1][b] + src.cls_len[2][b] + i;
    const uint4* ks = reinterpret_cast<const uint4*>(static_cast<const uint16_t*>(src.k16) + r * row_elems);
    const uint4* vs = reinterpret_cast<const uint4*>(static_cast<const uint16_t*>(src.v16) + r * row_elems);
    uint4* kd = reinterpret_cast<uint4*>(static_cast<uint16_t*>(dst.k16) + d * row_elems);
    uint4* vd = reinterpret_cast<uint4*>(static_cast<uint16_t*>(dst.v16) + d * row_elems);
    for (int e = threadIdx.x; e < row_elems / 8; e += 256) {
        kd[e] = ks[e];
        vd[e] = vs[e];
    }
}

template <int HD>
int run_dequantize(wq_ctx* ctx, int B, const wq_packed_kv* src, const wq_packed_kv* dst)
{
    hipStream_t st = ctx->stream;
    hipLaunchKernelGGL(k_dense_plan, dim3(1), dim3(256), 0, st, B, *src, *dst, wq_status_ptr(ctx));
    const dim3 blk(256);
    if (src->cap[0] > 0) hipLaunchKernelGGL((k_dequantize<HD, 2>), dim3((unsigned)(src->cap[0] / 32), src->Hkv), blk, 0, st, B, *src, *dst);
    if (src->cap[1] > 0) hipLaunchKernelGGL((k_dequantize<HD, 4>), dim3((unsigned)(src->cap[1] / 32), src->Hkv), blk, 0, st, B, *src, *dst);
    if (src->cap[2] > 0) hipLaunchKernelGGL((k_dequantize<HD, 8>), dim3((unsigned)(src->cap[2] / 32), src->Hkv), blk, 0, st, B, *src, *dst);
    if (src->cap16 > 0) hipLaunchKernelGGL(k_dense_copy, dim3((unsigned)src->cap16), blk, 0, st, B, src->Hkv * HD, *src, *dst);
    WQ_HIP_CHECK(ctx, hipGetLastError());
    return WQ_OK;
}

template <typename T, int HD>
int run(wq_ctx* ctx, const void* K_, const void* V_, int B, const int32_t* kv_off, const int32_t* win_size,
        const int32_t* win_off, const int32_t* perm, const int32_t* seg_windows, int64_t total_rows, const wq_packed_kv* pk)
{
    const T* K = static_cast<const T*>(K_);
    const T* V = static_cast<const T*>(V_);
    hipStream_t st = ctx->stream;
    int32_t* pre16 = reinterpret_cast<int32_t*>(ctx->ws + WQ_WS_HEADER);
    hipLaunchKernelGGL(k_plan, dim3(1), dim3(256), 0, st, B, kv_off, win_size, win_off, seg_windows, *pk, pre16,
                       wq_status_ptr(ctx));
    const int64_t n0 = pk->cap[0] / 32 * pk->Hkv, n1 = n0 + pk->cap[1] / 32 * pk->Hkv, n2 = n1 + pk->cap[2] / 32 * pk->Hkv;
    const int64_t rows16 = pk->cap16 > 0 ? (total_rows < pk->cap16 ? total_rows : pk->cap16) : 0;
    if (n2 + rows16 > 0x7FFFFFFF) return wq_fail(ctx, WQ_ERR_UNSUPPORTED, "too many blocks for one launch");
    if (n2 + rows16 > 0)
        hipLaunchKernelGGL((k_quantize_all<T, HD>), dim3((unsigned)(n2 + rows16)), dim3(256), 0, st, K, V, B, pk->group, kv_off, win_size,
                           win_off, perm, seg_windows, pre16, *pk, (unsigned)n0, (unsigned)n1, (unsigned)n2, wq_status_ptr(ctx));
    if (B > 0) hipLaunchKernelGGL(k_v_scale_max, dim3((unsigned)B * WQ_VS_PARTS), dim3(256), 0, st, B, *pk);
    WQ_HIP_CHECK(ctx, hipGetLastError());
    return WQ_OK;
}

}  // namespace

int wq_launch_append(wq_ctx* ctx, const void* k_new, const void* v_new, int dtype, int B, const wq_packed_kv* kv)
{
    const int row_elems = kv->Hkv * kv->hd;
    hipStream_t st = ctx->stream;
    switch (dtype) {
        case WQ_F32:
            hipLaunchKernelGGL(k_append16<float>, dim3(B), dim3(256), 0, st, static_cast<const float*>(k_new),
                               static_cast<const float*>(v_new), row_elems, *kv, wq_status_ptr(ctx));
            break;
        case WQ_BF16:
            hipLaunchKernelGGL(k_append16<__hip_bfloat16>, dim3(B), dim3(256), 0, st, static_cast<const __hip_bfloat16*>(k_new),
                               static_cast<const __hip_bfloat16*>(v_new), row_elems, *kv, wq_status_ptr(ctx));
            break;
        default:
            hipLaunchKernelGGL(k_append16<__half>, dim3(B), dim3(256), 0, st, static_cast<const __half*>(k_new),
                               static_cast<const __half*>(v_new), row_elems, *kv, wq_status_ptr(ctx));
    }
    WQ_HIP_CHECK(ctx, hipGetLastError());
    return WQ_OK;
}

int wq_launch_dequantize(wq_ctx* ctx, int B, const wq_packed_kv* src, const wq_packed_kv* dst)
{
    if (src->hd == 64 && src->group == 128) return wq_fail(ctx, WQ_ERR_UNSUPPORTED, "group larger than hd");
    return src->hd == 128 ? run_dequantize<128>(ctx, B, src, dst) : run_dequantize<64>(ctx, B, src, dst);
}

int wq_launch_quantize(wq_ctx* ctx, const void* K, const void* V, int dtype, int B, const int32_t* kv_off,
                       const int32_t* win_size, const int32_t* win_off, const int32_t* perm,
                       const int32_t* seg_windows, int64_t total_rows, const wq_packed_kv* out)
{
    if (out->hd == 64 && out->group == 128) return wq_fail(ctx, WQ_ERR_UNSUPPORTED, "group larger than hd");
#define WQ_RUN(T)                                                                                                   \
    (out->hd == 128 ? run<T, 128>(ctx, K, V, B, kv_off, win_size, win_off, perm, seg_windows, total_rows, out)      \
                    : run<T, 64>(ctx, K, V, B, kv_off, win_size, win_off, perm, seg_windows, total_rows, out))
    switch (dtype) {
        case WQ_F32: return WQ_RUN(float);
        case WQ_BF16: return WQ_RUN(__hip_bfloat16);
        default: return WQ_RUN(__half);
    }
#undef WQ_RUN
}
