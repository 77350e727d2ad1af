// a4: decode attention over the packed mixed-precision cache (Alg. 2 decode half; Sec. 3.3.2 shows that the
// block order does not matter without a mask, which is also what makes the split over tokens legal).
//
// One workgroup per (split, KV head, sequence) walks its share of the 2-, 4-, 8- and 16-bit segments with an
// online softmax (running max m, running sum l, unnormalised accumulator), writes one partial (m, l, acc) per
// query head; k_combine merges the partials of all splits by log-sum-exp in split order.  No float atomics:
// the result is deterministic for a given split count.
//
// k_decode_generic: plain vector-ALU kernel that reads codes field by field from the storage layout.  It
// handles every supported (hd, group) and is the reference implementation inside the library; the
// matrix-core body in wq_decode_mfma.h is the fast path for hd/group == 2.
#include <stdlib.h>

#include <type_traits>

#include "wq_internal.h"

namespace {

struct DecodeArgs {
    const void* q;
    int q_dtype;
    int B, Hq, rep, splits;
    float sm_scale;
    int splits16, nparts;   // workgroups on the 16-bit segment; nparts = splits + splits16 partials per (b, KV head)
    int use_mfma;
    int mfma16;             // the matrix-core kernel also walks the 16-bit segment
    int fused;              // the matrix-core kernel merges the splits itself (last workgroup per (b, KV head))
    unsigned* arrive;       // [B*Hkv] arrival counters, WQ_ARRIVE_STRIDE words apart, zero between launches
    int fixed_shares;       // every wavefront of the matrix-core kernel gets a fixed share of its workgroup's range
    wq_packed_kv kv;
    float* part;            // [B][Hkv][nparts][rep][hd + 2]
    float* out;
    float* lse;
    // appending one generated token per sequence in the same launch (matrix-core kernel, merged splits only):
    const uint16_t* k_new;  // [B][Hkv][hd] in the cache's 16-bit type, or NULL
    const uint16_t* v_new;
    uint32_t* status;       // device status word (a full 16-bit segment is reported there)
    float len_scale;        // > 0: a (sequence, KV head) with n tokens uses ceil(n * len_scale) of the launch's splits (at least one)
#ifdef WQ_TIMELINE
    long long* dbg;
#endif
};

// ---- the weights of the splits -----------------------------------------------------------------------------
// Reductions over the 64 lanes of a wavefront in a fixed order: four rotations inside the rows of 16 lanes (one
// data-parallel-primitive instruction each, no LDS), then the four rows' results as scalars.
template <int CTRL>
__device__ __forceinline__ float lanes_moved(float x)
{
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), CTRL, 0xF, 0xF, false));
}
__device__ __forceinline__ float lane_value(float x, int l)
{
    return __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, x), l));
}
__device__ __forceinline__ float wave_max(float x)
{
    x = fmaxf(x, lanes_moved<0x128>(x));           // row_ror:8, 4, 2, 1
    x = fmaxf(x, lanes_moved<0x124>(x));
    x = fmaxf(x, lanes_moved<0x122>(x));
    x = fmaxf(x, lanes_moved<0x121>(x));
    return fmaxf(fmaxf(lane_value(x, 0), lane_value(x, 16)), fmaxf(lane_value(x, 32), lane_value(x, 48)));
}
__device__ __forceinline__ float wave_sum(float x)
{
    x += lanes_moved<0x128>(x);
    x += lanes_moved<0x124>(x);
    x += lanes_moved<0x122>(x);
    x += lanes_moved<0x121>(x);
    return (lane_value(x, 0) + lane_value(x, 16)) + (lane_value(x, 32) + lane_value(x, 48));
}

// Up to 64 splits, one per lane: lane s holds m_s (-inf beyond the last split) and l_s; it gets its weight
// w_s = e^{m_s - M}, and every lane M = max m_s and L = sum l_s w_s.  Both merges (the one inside the matrix-core
// kernel and k_combine) go through this function when there are at most 64 splits and then sum the numerators in
// split order, which is why their results agree bit for bit.
__device__ __forceinline__ void merge_weights_lanes(float m, float l, float& w, float& M, float& L)
{
    M = wave_max(m);
    w = (m == -INFINITY) ? 0.f : __expf(m - M);
    L = wave_sum(l * w);
}

// More than 64 splits (k_combine only): one wavefront turns the m_s of n splits (in w) into the weights in place and
// returns M and L.  Lane i takes the splits i, i + 64, ..., then the lanes are reduced as above.
__device__ __forceinline__ void merge_weights(float* w, const float* l, int n, float& M, float& L)
{
    const int lane = threadIdx.x & 63;
    float mx = -INFINITY;
    for (int s = lane; s < n; s += 64) mx = fmaxf(mx, w[s]);
    mx = wave_max(mx);
    float sum = 0.f;
    for (int s = lane; s < n; s += 64) {
        const float ms = w[s];
        const float e = (ms == -INFINITY) ? 0.f : __expf(ms - mx);
        w[s] = e;
        sum = fmaf(l[s], e, sum);
    }
    M = mx;
    L = wave_sum(sum);
}

__device__ __forceinline__ float load_q(const void* q, int dtype, int64_t i)
{
    if (dtype == WQ_F32) return static_cast<const float*>(q)[i];
    if (dtype == WQ_BF16) return wq_bf16_bits_to_float(static_cast<const uint16_t*>(q)[i]);
    return wq_f16_bits_to_float(static_cast<const uint16_t*>(q)[i]);
}

}  // namespace

#include "wq_decode_mfma.h"

namespace {

// field n (BITS wide) of a little-endian packed byte image
template <int BITS>
__device__ __forceinline__ int field(const uint8_t* base, int64_t n)
{
    int64_t bit = n * BITS;
    return (base[bit >> 3] >> (bit & 7)) & ((1 << BITS) - 1);
}

template <int HD>
struct Smem {
    float q[WQ_MAX_REP][HD];
    float logit[WQ_MAX_REP][32];
    float p[WQ_MAX_REP][32];
    float red[256 / HD][WQ_MAX_REP][HD];
    float m[WQ_MAX_REP], l[WQ_MAX_REP], scale[WQ_MAX_REP];
};

// One 32-token step: logits are in sm.logit (-inf for invalid tokens).  Thread (r = tid/32, u = tid%32) owns one
// (head, token) pair: block max and sum by wavefront shuffles inside its 32 lanes, running (m, l) in LDS; leaves the
// weights in sm.p and rescales every thread's accumulators.
template <int HD>
__device__ __forceinline__ void softmax_step(Smem<HD>& sm, int rep, float* acc)
{
    const int tid = threadIdx.x;
    const int r = tid >> 5, u = tid & 31;
    const float lg = r < rep ? sm.logit[r][u] : -INFINITY;
    float bm = lg;
#pragma unroll
    for (int o = 16; o > 0; o >>= 1) bm = fmaxf(bm, __shfl_xor(bm, o, 64));
    const float mo = sm.m[r];
    const float mn = fmaxf(mo, bm);
    const float p = (mn == -INFINITY) ? 0.f : __expf(lg - mn);
    float ps = p;
#pragma unroll
    for (int o = 16; o > 0; o >>= 1) ps += __shfl_xor(ps, o, 64);
    sm.p[r][u] = p;
    __syncthreads();                      // every lane has read the old m before it changes
    if (u == 0) {
        const float sc = (mn == -INFINITY) ? 1.0f : __expf(mo - mn);
        sm.scale[r] = sc;
        sm.m[r] = mn;
        sm.l[r] = sm.l[r] * sc + ps;
    }
    __syncthreads();
#pragma unroll
    for (int k = 0; k < WQ_MAX_REP; k++) acc[k] *= sm.scale[k];
}

template <int HD, int BITS>
__device__ void walk_class(const DecodeArgs& a, Smem<HD>& sm, int b, int kvh, int share, int nshare, float* acc)
{
    constexpr int C = BITS == 2 ? 0 : (BITS == 4 ? 1 : 2);
    constexpr int Q = HD / 4, CT = HD / 16, PARTS = 256 / HD;
    const wq_packed_kv& kv = a.kv;
    const int tid = threadIdx.x;
    const int G = HD / kv.group;
    const int len = kv.cls_len[C][b];
    const int nblk = (len + 31) / 32;
    const int blk_lo = (int)((int64_t)share * nblk / nshare), blk_hi = (int)((int64_t)(share + 1) * nblk / nshare);
    const int64_t tok_base = kv.cls_off[C][b];
    const int64_t cap = kv.cap[C];
    const uint8_t* kcodes = static_cast<const uint8_t*>(kv.codes[C]) + (int64_t)kvh * cap * HD * BITS / 8;
    const uint8_t* vcodes = static_cast<const uint8_t*>(kv.codes[C]) + ((int64_t)kv.Hkv + kvh) * cap * HD * BITS / 8;
    const uint32_t* kmeta = static_cast<const uint32_t*>(kv.meta[C]) + (int64_t)kvh * cap * G;
    const uint32_t* vmeta = static_cast<const uint32_t*>(kv.meta[C]) + ((int64_t)kv.Hkv + kvh) * cap * G;

    for (int blk = blk_lo; blk < blk_hi; blk++) {
        const int64_t t0 = tok_base + (int64_t)blk * 32;       // absolute token slot of the block
        // ---- logits: thread = (token u, eighth p of the channels) ----
        {
            const int u = tid >> 3, p = tid & 7;
            const int64_t t = t0 + u;
            const int64_t tile = t >> 4;
            const int mrow = (int)(t & 15);
            const uint8_t* tb = kcodes + tile * (16 * HD * BITS / 8);
            float part[WQ_MAX_REP];
#pragma unroll
            for (int r = 0; r < WQ_MAX_REP; r++) part[r] = 0.f;
            for (int i = 0; i < HD / 8; i++) {
                int ch = p * (HD / 8) + i;
                int j = ch / Q, e = ch % Q;
                int code = field<BITS>(tb, (int64_t)(j * 16 + mrow) * Q + e);
                uint32_t w = kmeta[(tile * G + ch / kv.group) * 16 + mrow];
                float kh = fmaf(wq_f16_bits_to_float(w & 0xFFFF), (float)code, wq_f16_bits_to_float(w >> 16));
#pragma unroll
                for (int r = 0; r < WQ_MAX_REP; r++)
                    if (r < a.rep) part[r] = fmaf(sm.q[r][ch], kh, part[r]);
            }
#pragma unroll
            for (int r = 0; r < WQ_MAX_REP; r++) {
                float v = part[r];
                v += __shfl_xor(v, 1, 64);
                v += __shfl_xor(v, 2, 64);
                v += __shfl_xor(v, 4, 64);
                if (p == 0 && r < a.rep) sm.logit[r][u] = (blk * 32 + u < len) ? v * a.sm_scale : -INFINITY;
            }
        }
        __syncthreads();
        softmax_step<HD>(sm, a.rep, acc);
        // ---- values: thread = (channel c, token part tp) ----
        {
            const int c = tid % HD, tp = tid / HD;
            const int ct = c / 16, mm = c % 16;
            const uint8_t* vb = vcodes + (t0 >> 5) * (32 * HD * BITS / 8);
            for (int u = tp * (32 / PARTS); u < (tp + 1) * (32 / PARTS); u++) {
                int jj = (u % 16) / 4, tau = 4 * (u / 16) + u % 4;
                int code = field<BITS>(vb, ((int64_t)(jj * 16 + mm) * CT + ct) * 8 + tau);
                const int64_t t = t0 + u;
                uint32_t w = vmeta[((t >> 4) * G + c / kv.group) * 16 + (t & 15)];
                float vh = fmaf(wq_f16_bits_to_float(w & 0xFFFF), (float)code, wq_f16_bits_to_float(w >> 16));
#pragma unroll
                for (int r = 0; r < WQ_MAX_REP; r++)
                    if (r < a.rep) acc[r] = fmaf(sm.p[r][u], vh, acc[r]);
            }
        }
        __syncthreads();
    }
}

template <int HD>
__device__ void walk_seg16(const DecodeArgs& a, Smem<HD>& sm, int b, int kvh, int share, int nshare, float* acc)
{
    constexpr int PARTS = 256 / HD;
    const wq_packed_kv& kv = a.kv;
    const int tid = threadIdx.x;
    const int len = kv.len16[b];
    const int nblk = (len + 31) / 32;
    const int blk_lo = (int)((int64_t)share * nblk / nshare), blk_hi = (int)((int64_t)(share + 1) * nblk / nshare);
    const uint16_t* k16 = static_cast<const uint16_t*>(kv.k16);
    const uint16_t* v16 = static_cast<const uint16_t*>(kv.v16);
    const bool bf = kv.dtype16 == WQ_BF16;
    for (int blk = blk_lo; blk < blk_hi; blk++) {
        {
            const int u = tid >> 3, p = tid & 7;
            const int i = blk * 32 + u;
            const bool valid = i < len;
            const int64_t row = ((int64_t)kv.off16[b] + (valid ? i : 0)) * kv.Hkv + kvh;
            float part[WQ_MAX_REP];
#pragma unroll
            for (int r = 0; r < WQ_MAX_REP; r++) part[r] = 0.f;
            for (int k = 0; k < HD / 8; k++) {
                int ch = p * (HD / 8) + k;
                uint32_t h = valid ? k16[row * HD + ch] : 0;
                float kh = bf ? wq_bf16_bits_to_float(h) : wq_f16_bits_to_float(h);
#pragma unroll
                for (int r = 0; r < WQ_MAX_REP; r++)
                    if (r < a.rep) part[r] = fmaf(sm.q[r][ch], kh, part[r]);
            }
#pragma unroll
            for (int r = 0; r < WQ_MAX_REP; r++) {
                float v = part[r];
                v += __shfl_xor(v, 1, 64);
                v += __shfl_xor(v, 2, 64);
                v += __shfl_xor(v, 4, 64);
                if (p == 0 && r < a.rep) sm.logit[r][u] = valid ? v * a.sm_scale : -INFINITY;
            }
        }
        __syncthreads();
        softmax_step<HD>(sm, a.rep, acc);
        {
            const int c = tid % HD, tp = tid / HD;
            for (int u = tp * (32 / PARTS); u < (tp + 1) * (32 / PARTS); u++) {
                const int i = blk * 32 + u;
                if (i >= len) break;
                const int64_t row = ((int64_t)kv.off16[b] + i) * kv.Hkv + kvh;
                uint32_t h = v16[row * HD + c];
                float vh = bf ? wq_bf16_bits_to_float(h) : wq_f16_bits_to_float(h);
#pragma unroll
                for (int r = 0; r < WQ_MAX_REP; r++)
                    if (r < a.rep) acc[r] = fmaf(sm.p[r][u], vh, acc[r]);
            }
        }
        __syncthreads();
    }
}

template <int HD>
__device__ void decode_generic_body(const DecodeArgs& a, void* smem_raw, bool quantized, int share, int nshare, int part_idx)
{
    Smem<HD>& sm = *reinterpret_cast<Smem<HD>*>(smem_raw);
    const int kvh = blockIdx.y, b = blockIdx.z;
    const int tid = threadIdx.x;
    for (int i = tid; i < a.rep * HD; i += 256) {
        int r = i / HD, ch = i % HD;
        sm.q[r][ch] = load_q(a.q, a.q_dtype, ((int64_t)b * a.Hq + kvh * a.rep + r) * HD + ch);
    }
    __syncthreads();
    if (tid < WQ_MAX_REP) {
        sm.m[tid] = -INFINITY;
        sm.l[tid] = 0.f;
        sm.scale[tid] = 1.f;
    }
    __syncthreads();
    float acc[WQ_MAX_REP];
#pragma unroll
    for (int r = 0; r < WQ_MAX_REP; r++) acc[r] = 0.f;
    if (quantized) {
        walk_class<HD, 2>(a, sm, b, kvh, share, nshare, acc);
        walk_class<HD, 4>(a, sm, b, kvh, share, nshare, acc);
        walk_class<HD, 8>(a, sm, b, kvh, share, nshare, acc);
    }
    walk_seg16<HD>(a, sm, b, kvh, share, nshare, acc);

    // reduce the token parts, write the partial
    constexpr int PARTS = 256 / HD;
    const int c = tid % HD, tp = tid / HD;
#pragma unroll
    for (int r = 0; r < WQ_MAX_REP; r++)
        if (r < a.rep) sm.red[tp][r][c] = acc[r];
    __syncthreads();
    float* out = a.part + (((int64_t)b * a.kv.Hkv + kvh) * a.nparts + part_idx) * a.rep * (HD + 2);
    if (tp == 0) {
        for (int r = 0; r < a.rep; r++) {
            float s = 0.f;
            for (int k = 0; k < PARTS; k++) s += sm.red[k][r][c];
            out[r * (HD + 2) + c] = s;
        }
    }
    if (tid < a.rep) {
        out[tid * (HD + 2) + HD] = sm.m[tid];
        out[tid * (HD + 2) + HD + 1] = sm.l[tid];
    }
}

// Generic kernel: every segment (use_mfma == 0), or only the 16-bit segment next to a matrix-core launch, in
// which case its partials follow the matrix-core ones (slot splits + x).
template <int HD>
__global__ __launch_bounds__(256) void k_decode_generic(DecodeArgs a)
{
    __shared__ __align__(16) unsigned char smem[sizeof(Smem<HD>)];
    const int x = blockIdx.x;
    if (!a.use_mfma)
        decode_generic_body<HD>(a, smem, true, x, a.splits, x);
    else
        decode_generic_body<HD>(a, smem, false, x, a.splits16, a.splits + x);
}

// Matrix-core kernel: the quantized classes of one (split, KV head, sequence).
template <int HD>
__global__ __launch_bounds__(64 * WQ_WAVES) void k_decode_mfma(DecodeArgs a)
{
    __shared__ __align__(16) unsigned char smem[sizeof(MfmaSmem<HD>)];
    wq_decode_mfma_body<HD>(a, smem);
}

// out[b,h,:] = sum_s acc_s e^{m_s - M} / sum_s l_s e^{m_s - M},  M = max_s m_s;  lse = M + log(sum).
// One workgroup per (b, h); the weights come from merge_weights (first wavefront), the numerators are summed in split
// order with all loads of a thread independent of each other (no data-dependent control flow around them): the same
// arithmetic in the same order as the merge inside the matrix-core kernel.
__global__ __launch_bounds__(128) void k_combine(const float* __restrict__ part, int Hq, int rep, int nparts, int hd,
                                                 float* __restrict__ out, float* __restrict__ lse)
{
    __shared__ float s_w[1024 + 32];
    __shared__ float s_l[1024 + 32];
    __shared__ float s_red[2];
    const int h = blockIdx.x, b = blockIdx.y;
    const int kvh = h / rep, r = h % rep;
    const int Hkv = Hq / rep;
    const int tid = threadIdx.x;
    const int64_t stride = (int64_t)rep * (hd + 2);
    const float* base = part + (((int64_t)b * Hkv + kvh) * nparts) * stride + (int64_t)r * (hd + 2);
    constexpr int CHUNK = 32;
    float pre[CHUNK];                      // this channel's numerators of the first CHUNK splits: in flight while the weights are found
#pragma unroll
    for (int k = 0; k < CHUNK; k++) pre[k] = (k < nparts && tid < hd) ? base[(int64_t)k * stride + tid] : 0.f;
    for (int s = tid; s < nparts; s += 128) {
        s_w[s] = base[s * stride + hd];
        s_l[s] = base[s * stride + hd + 1];
    }
    __syncthreads();
    if (tid < 64) {
        float M, L;
        if (nparts <= 64) {
            float w;
            merge_weights_lanes(tid < nparts ? s_w[tid] : -INFINITY, tid < nparts ? s_l[tid] : 0.f, w, M, L);
            if (tid < nparts) s_w[tid] = w;
        } else {
            merge_weights(s_w, s_l, nparts, M, L);
        }
        if (tid == 0) {
            s_red[0] = M;
            s_red[1] = L;
        }
    }
    __syncthreads();
    const float M = s_red[0], L = s_red[1];
    float acc = 0.f;
#pragma unroll
    for (int k = 0; k < CHUNK; k++) acc = fmaf(pre[k], k < nparts ? s_w[k] : 0.f, acc);
    if (tid < hd) {
        for (int s0 = CHUNK; s0 < nparts; s0 += CHUNK) {
            float v[CHUNK];
#pragma unroll
            for (int k = 0; k < CHUNK; k++) v[k] = (s0 + k < nparts) ? base[(int64_t)(s0 + k) * stride + tid] : 0.f;
#pragma unroll
            for (int k = 0; k < CHUNK; k++) acc = fmaf(v[k], (s0 + k < nparts) ? s_w[s0 + k] : 0.f, acc);
        }
        out[((int64_t)b * Hq + h) * hd + tid] = L > 0.f ? acc / L : 0.f;
    }
    if (lse && tid == 0) lse[(int64_t)b * Hq + h] = L > 0.f ? M + logf(L) : -INFINITY;
}

}  // namespace

// workgroups per (sequence, KV head) given to the 16-bit segment by the matrix-core launch: about one per
// 32 rows of the average sequence's capacity, between 1 and 32
static int wq_decode_splits16(int B, int64_t cap16)
{
    int64_t per = B > 0 ? cap16 / B : 0;
    int64_t n = (per + 31) / 32;
    return (int)(n < 1 ? 1 : (n > 32 ? 32 : n));
}

size_t wq_decode_ws_bytes(int B, int Hq, int hd, int splits)
{
    if (B <= 0 || Hq <= 0 || hd <= 0 || splits <= 0) return 0;
    return wq_align256(sizeof(float) * (size_t)B * Hq * (splits + 32) * (hd + 2));
}

// Can wq_launch_decode append k_new, v_new (element type new_dtype) itself with these arguments?  Only the matrix-core
// kernel that walks every segment and merges its splits does: it needs the new rows in the cache's own 16-bit type
// and one more counter per sequence in the workspace header.
bool wq_decode_can_append(int q_dtype, int B, int Hq, const wq_packed_kv* kv, int num_splits, int algo, int new_dtype)
{
    if (algo & (WQ_DECODE_PARTIALS_ONLY | WQ_DECODE_SEPARATE_MERGE)) return false;
    const int balgo = algo & ~WQ_DECODE_FLAGS;
    const bool use_mfma = (balgo == WQ_DECODE_MFMA) || (balgo == WQ_DECODE_AUTO && kv->hd / kv->group == 2);
    const bool mfma16 = use_mfma && !(kv->dtype16 == WQ_BF16 && q_dtype != WQ_BF16);
    const int rep = Hq / kv->Hkv;
    return mfma16 && new_dtype == kv->dtype16 && (int64_t)B * kv->Hkv + B <= WQ_MAX_ARRIVE && num_splits <= WQ_MAX_FUSED_SPLITS &&
           rep <= WQ_MAX_REP;
}

int wq_launch_decode(wq_ctx* ctx, const void* q, int q_dtype, int B, int Hq, const wq_packed_kv* kv, float sm_scale,
                     int num_splits, int algo, float* out, float* lse, const void* k_new, const void* v_new,
                     int64_t longest_tokens)
{
    const bool partials_only = (algo & WQ_DECODE_PARTIALS_ONLY) != 0;
    const bool fixed_shares = (algo & WQ_DECODE_FIXED_SHARES) != 0;
    const bool separate_merge = (algo & WQ_DECODE_SEPARATE_MERGE) != 0;
    algo &= ~WQ_DECODE_FLAGS;
    DecodeArgs a;
    a.q = q;
    a.q_dtype = q_dtype;
    a.B = B;
    a.Hq = Hq;
    a.rep = Hq / kv->Hkv;
    a.splits = num_splits;
    a.sm_scale = sm_scale;
    a.use_mfma = (algo == WQ_DECODE_MFMA) || (algo == WQ_DECODE_AUTO && kv->hd / kv->group == 2);
    // a bf16 cache needs the exact bf16 query for the bf16 instruction; other query types send the 16-bit
    // segment to the generic kernel
    a.mfma16 = a.use_mfma && !(kv->dtype16 == WQ_BF16 && q_dtype != WQ_BF16);
    a.splits16 = (a.use_mfma && !a.mfma16) ? wq_decode_splits16(B, kv->cap16) : 0;
    a.nparts = a.splits + a.splits16;
    a.kv = *kv;
    a.fixed_shares = fixed_shares;
    a.arrive = reinterpret_cast<unsigned*>(ctx->ws + 256);
    // one launch does it all when the matrix-core kernel walks every segment, the counters fit the workspace
    // header and a wavefront's lanes hold the splits' weights
    a.fused = a.use_mfma && a.mfma16 && !partials_only && !separate_merge && (int64_t)B * kv->Hkv <= WQ_MAX_ARRIVE &&
              a.nparts <= WQ_MAX_FUSED_SPLITS;
    // the shares of the token axis are cut on a 32-bit cost axis (at most 500 per 32-token block)
    if (a.use_mfma && (int64_t)kv->cap[0] + kv->cap[1] + kv->cap[2] + kv->cap16 > ((int64_t)1 << 27))
        return wq_fail(ctx, WQ_ERR_UNSUPPORTED, "the matrix-core decode kernel takes caches of up to 2^27 token slots");
    a.part = reinterpret_cast<float*>(ctx->ws + WQ_WS_HEADER);
    a.out = out;
    a.k_new = static_cast<const uint16_t*>(k_new);
    a.v_new = static_cast<const uint16_t*>(v_new);
    a.status = wq_status_ptr(ctx);
    if (k_new && !a.fused) return wq_fail(ctx, WQ_ERR_UNSUPPORTED, "this decode launch cannot append");
    // splits by length: only where the kernel merges the splits itself (the separate merge kernel reads every partial)
    a.len_scale = (a.fused && longest_tokens > 0) ? (float)a.splits / (float)longest_tokens : 0.f;
#ifdef WQ_TIMELINE
    a.dbg = getenv("WQ_TIMELINE") ? reinterpret_cast<long long*>(ctx->ws + ctx->ws_bytes - (8 << 20)) : nullptr;
#endif
    a.lse = lse;
    const dim3 blk(256);
    const dim3 grid_q(a.splits, kv->Hkv, B), grid_16(a.splits16 > 0 ? a.splits16 : 1, kv->Hkv, B);
    // the matrix-core kernel maps workgroups (of WQ_WAVES wavefronts) to units itself
    const dim3 grid_m((unsigned)kv->Hkv, (unsigned)B, (unsigned)a.splits), blk_m(64 * WQ_WAVES);
    const int tslot = (int)(ctx->ev_calls % WQ_TIMING_RING);
    if (ctx->timing) (void)hipEventRecord(ctx->ev[2 * tslot], ctx->stream);
    if (kv->hd == 128) {
        if (a.use_mfma) {
            hipLaunchKernelGGL(k_decode_mfma<128>, grid_m, blk_m, 0, ctx->stream, a);
            if (ctx->timing) (void)hipEventRecord(ctx->ev[2 * tslot + 1], ctx->stream);
            if (a.splits16 > 0) hipLaunchKernelGGL(k_decode_generic<128>, grid_16, blk, 0, ctx->stream, a);
        } else {
            hipLaunchKernelGGL(k_decode_generic<128>, grid_q, blk, 0, ctx->stream, a);
            if (ctx->timing) (void)hipEventRecord(ctx->ev[2 * tslot + 1], ctx->stream);
        }
    } else {
        if (a.use_mfma) {
            hipLaunchKernelGGL(k_decode_mfma<64>, grid_m, blk_m, 0, ctx->stream, a);
            if (ctx->timing) (void)hipEventRecord(ctx->ev[2 * tslot + 1], ctx->stream);
            if (a.splits16 > 0) hipLaunchKernelGGL(k_decode_generic<64>, grid_16, blk, 0, ctx->stream, a);
        } else {
            hipLaunchKernelGGL(k_decode_generic<64>, grid_q, blk, 0, ctx->stream, a);
            if (ctx->timing) (void)hipEventRecord(ctx->ev[2 * tslot + 1], ctx->stream);
        }
    }
    if (!partials_only && !a.fused)
        hipLaunchKernelGGL(k_combine, dim3(Hq, B), dim3(128), 0, ctx->stream, a.part, Hq, a.rep, a.nparts, kv->hd, out, lse);
    if (ctx->timing) ctx->ev_calls++;
    WQ_HIP_CHECK(ctx, hipGetLastError());
    return WQ_OK;
}
