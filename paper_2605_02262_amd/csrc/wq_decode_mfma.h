// a4, matrix-core path: decode attention over the packed cache for hd/group == 2 (Alg. 2 decode half).
// (included by wq_decode.hip, after DecodeArgs and load_q)
//
// One wavefront walks 32-token blocks of a class on its own (no workgroup barrier inside the loop):
//
//   S^T = K_codes . Q^T      v_mfma_f32_16x16x32_f16, A = 16 tokens x 32 contraction slots of raw codes,
//                            B = query heads.  The 16 output columns are (group g, head h): B is block-diagonal,
//                            slots 0..15 carry group-0 channels and feed columns 0..7, slots 16..31 carry group-1
//                            channels and feed columns 8..15, so one accumulator tile holds both groups' integer
//                            dot products and every lane of the softmax has real work (7 of 8 columns per half).
//   dequant                  logit = s0*D0 + m0*sum(q over group 0) + s1*D1 + m1*sum(q over group 1): each lane
//                            applies its own group's (s, m), the two halves meet with one DPP row rotate.
//   online softmax           reference exponent per column, shared by the wavefront's four lane groups.  It starts
//                            as the first block's largest logit and moves (with a rescale of the output
//                            accumulators) only when a logit exceeds it by more than 2^8: weights stay below
//                            2^8, far inside what f32 sums and the f16 operand hold, and a new largest logit
//                            (there is one in most blocks of a short walk) costs nothing.
//   O^T += V_codes^T . P'^T  P' = p * s_v (per value group, hence the same 16 columns), raw V codes as A; the
//                            m_v part of the dequantised values is the scalar sum  p * m_v  kept per lane.
//
// Codes go into the f16 operands without arithmetic: a b-bit field masked in place inside a 16-bit half is the
// f16 subnormal  code * 2^(shift-24), which the matrix cores consume exactly; the per-slot power of two is
// folded into the other operand (q or P'), the common 2^-24 into constants applied after the contraction.
//
// The storage layout (wq.h) is exactly the per-lane operand order, so every load is one contiguous piece per
// lane, a whole tile per wavefront.  Scales and minima travel as one coalesced word per lane and block and are
// redistributed through LDS.  Each wavefront builds the query operands of the class it walks from global memory.
#pragma once

#ifdef WQ_TIMELINE   // development aid: per-workgroup phase time stamps (100 MHz clock) at the end of the workspace
#define WQ_WG ((int64_t)(blockIdx.z * gridDim.y + blockIdx.y) * gridDim.x + blockIdx.x)
#define WQ_STAMP(k) do { if (a.dbg && threadIdx.x == 0) a.dbg[WQ_WG * 64 + (k)] = wall_clock64(); } while (0)
#define WQ_WSTAMP(k, val) do { if (a.dbg && (threadIdx.x & 63) == 0) a.dbg[WQ_WG * 64 + 8 + (threadIdx.x >> 6) * 6 + (k)] = (val); } while (0)
#else
#define WQ_STAMP(k) do { } while (0)
#define WQ_WSTAMP(k, val) do { } while (0)
#endif

namespace {

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef _Float16 half2v __attribute__((ext_vector_type(2)));
typedef float floatx4 __attribute__((ext_vector_type(4)));

struct U4 {
    uint32_t x, y, z, w;
};

__device__ __forceinline__ half8 as_half8(uint32_t a, uint32_t b, uint32_t c, uint32_t d)
{
    U4 u{a, b, c, d};
    return __builtin_bit_cast(half8, u);
}

__device__ __forceinline__ floatx4 mfma(half8 a, half8 b, floatx4 c)
{
    return __builtin_amdgcn_mfma_f32_16x16x32_f16(a, b, c, 0, 0, 0);
}

__device__ __forceinline__ float f16lo(uint32_t w) { return wq_f16_bits_to_float(w & 0xFFFFu); }
__device__ __forceinline__ float f16hi(uint32_t w) { return wq_f16_bits_to_float(w >> 16); }

// largest of three without the quieting moves that fmaxf brings along (inputs here are never signalling NaNs)
__device__ __forceinline__ float max3(float a, float b, float c)
{
    float r;
    asm("v_max3_f32 %0, %1, %2, %3" : "=v"(r) : "v"(a), "v"(b), "v"(c));
    return r;
}

// (f16 in the low half of w) * p, rounded to f16, into the low / the high half of a register
__device__ __forceinline__ uint32_t mul_f16lo_to_lo(uint32_t w, float p)
{
    uint32_t r;
    asm("v_fma_mixlo_f16 %0, %1, %2, 0 op_sel_hi:[1,0,0]" : "=v"(r) : "v"(w), "v"(p));
    return r;
}
__device__ __forceinline__ uint32_t mul_f16lo_to_hi(uint32_t acc, uint32_t w, float p)
{
    asm("v_fma_mixhi_f16 %0, %1, %2, 0 op_sel_hi:[1,0,0]" : "+v"(acc) : "v"(w), "v"(p));
    return acc;
}

// rotate by 8 lanes inside each row of 16 lanes: lane (g,h) <-> lane (1-g,h)
__device__ __forceinline__ float ror8(float v)
{
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x128, 0xF, 0xF, false));
}

// ---- where contraction slot e (0..7) of k-step r finds its channel (inside the lane's quarter of hd/4
// channels) and the left shift its code keeps inside the f16 half; c = class index (0,1,2 = 2,4,8 bits) ----
__device__ __forceinline__ void k_slot(int c, int r, int e, int& ch, int& sh)
{
    const int v = e >> 1, hi = e & 1;
    if (c == 0) {               // dword d = r/2 holds 16 fields; pair p = 4*(r%2)+v is (field p, field p+8)
        const int d = r >> 1, p = 4 * (r & 1) + v;
        ch = 16 * d + p + 8 * hi;
        sh = p <= 4 ? 2 * p : 2 * (p - 5);
    } else if (c == 1) {        // dword r holds 8 fields; pair v is (field v, field v+4)
        ch = 8 * r + v + 4 * hi;
        sh = 4 * (v & 1);
    } else if (c == 2) {        // dwords 2r, 2r+1; register v = (dword v/2, bytes (v%2, v%2+2))
        const int d = 2 * r + (v >> 1);
        ch = 4 * d + (v & 1) + 2 * hi;
        sh = 0;
    } else {                    // 16-bit segment: elements in natural order
        ch = 8 * r + e;
        sh = 0;
    }
}

// unpack the K chunk of one lane (hd/4 codes of one token) into the A operand of k-step r
template <int BITS>
__device__ __forceinline__ half8 k_operand(const uint32_t* x, int r)
{
    if (BITS == 2) {
        const uint32_t w = x[r >> 1];
        if ((r & 1) == 0)
            return as_half8(w & 0x00030003u, w & 0x000C000Cu, w & 0x00300030u, w & 0x00C000C0u);
        const uint32_t y = w >> 10;
        return as_half8(w & 0x03000300u, y & 0x00030003u, y & 0x000C000Cu, y & 0x00300030u);
    } else if (BITS == 4) {
        const uint32_t w = x[r], y = w >> 8;
        return as_half8(w & 0x000F000Fu, w & 0x00F000F0u, y & 0x000F000Fu, y & 0x00F000F0u);
    } else {
        const uint32_t w0 = x[2 * r], w1 = x[2 * r + 1];
        return as_half8(w0 & 0x00FF00FFu, __builtin_amdgcn_perm(0u, w0, 0x0c030c01u), w1 & 0x00FF00FFu,
                        __builtin_amdgcn_perm(0u, w1, 0x0c030c01u));
    }
}

// power of two that P' carries in register v (slots 2v, 2v+1) so that V's in-place codes come out unscaled
template <int BITS>
__device__ __forceinline__ float v_slot_scale(int v)
{
    if (BITS == 2) return v == 0 ? 1.0f : (v == 1 ? 0.25f : (v == 2 ? 0.0625f : 0.015625f));
    if (BITS == 4) return (v & 1) ? 0.0625f : 1.0f;
    return 1.0f;
}

template <int BITS>
__device__ __forceinline__ float v_slot_shift(int v)      // -log2 of v_slot_scale
{
    if (BITS == 2) return 2.0f * (float)v;
    if (BITS == 4) return (v & 1) ? 4.0f : 0.0f;
    return 0.0f;
}

// unpack the V fragment of one lane (for channel tile ct: 8 tokens of one channel) into an A operand
template <int BITS>
__device__ __forceinline__ half8 v_operand(const uint32_t* x, int ct)
{
    if (BITS == 2) {            // dword ct/2: fields 0..7 = even tile, 8..15 = odd tile
        uint32_t y = __builtin_amdgcn_perm(0u, x[ct >> 1], 0x03010200u);   // bytes (b0,b2,b1,b3)
        if (ct & 1) y >>= 8;
        return as_half8(y & 0x00030003u, y & 0x000C000Cu, y & 0x00300030u, y & 0x00C000C0u);
    } else if (BITS == 4) {
        const uint32_t w = x[ct], y = w >> 8;
        return as_half8(w & 0x000F000Fu, w & 0x00F000F0u, y & 0x000F000Fu, y & 0x00F000F0u);
    } else {                    // dwords 2ct (tokens tau 0..3), 2ct+1 (tau 4..7)
        const uint32_t lo = x[2 * ct], hi = x[2 * ct + 1];
        return as_half8(__builtin_amdgcn_perm(hi, lo, 0x0c040c00u), __builtin_amdgcn_perm(hi, lo, 0x0c050c01u),
                        __builtin_amdgcn_perm(hi, lo, 0x0c060c02u), __builtin_amdgcn_perm(hi, lo, 0x0c070c03u));
    }
}

template <int HD>
struct WaveState {
    floatx4 O[HD / 16];   // O^T tiles: row = channel 16ct + 4j + i, column = (g,h)
    float m;              // reference exponent of this column (a recent largest logit), log2 domain, shared by the four lane groups
    float l;              // this lane's share of sum p
    float accM;           // this lane's share of sum p * m_v
    float up;             // log2 of the factor that the weights of the quantized classes are formed with (the same in all lanes)
};

// 32-token blocks in flight per wavefront and class: enough bytes to keep the memory system busy while a block
// is being worked on (a 2-bit block is 2.5 KB, an 8-bit block 8.5 KB)
constexpr int WQ_D2 = 4, WQ_D4 = 3, WQ_D8 = 2;
constexpr int WQ_TAPER_TICKETS = 16;   // the last blocks of a workgroup's range, two per wavefront, are walked with half the pipeline (measured: 0.45 us per call)
constexpr int WQ_FIRST_TICKETS = 4;    // blocks every wavefront starts with (the deepest pipeline's fill)
constexpr int WQ_WAVES = 8;            // wavefronts per workgroup: one workgroup per compute unit, two wavefronts per SIMD
constexpr float WQ_MAX_SLACK = 5.0f;   // log2 of the largest softmax weight tolerated before the reference exponent moves
// The weights meet the value scales in fp16 (P' = p * s_v).  They are formed 2^up too large (for free, in the exponent of
// the exp2), which the sums undo exactly at the end; up is chosen per sequence from its largest value scale s_max (a table
// of the cache that the quantizer fills) so that the largest product, 2^(WQ_MAX_SLACK + up) * s_max, lies in
// [2^(WQ_P_TOP - 1), 2^WQ_P_TOP]: nothing overflows whatever the values' magnitude, and a weight has to be
// 2^-(24 + WQ_P_TOP - WQ_MAX_SLACK - 6) = 2^-29 of the largest one, in a group whose scale is the sequence's largest and
// in the slot that is shifted most, before it is lost.
constexpr int WQ_P_TOP = 15;
// up for a sequence whose largest value scale is s_max (0: no quantized token; any up will do)
__device__ __forceinline__ float weight_upscale(float s_max)
{
    const uint32_t u = __float_as_uint(s_max);
    const int ceil_log2 = (int)((u >> 23) & 0xFFu) - 127 + ((u & 0x7FFFFFu) != 0u ? 1 : 0);
    const int up = (WQ_P_TOP - (int)WQ_MAX_SLACK) - ceil_log2;
    return s_max > 0.f ? (float)min(max(up, -16), 40) : 6.0f;
}
__device__ __forceinline__ float pow2_of(float e) { return __uint_as_float((uint32_t)(127 + (int)e) << 23); }   // e an integer in [-126, 127]
constexpr int VT_PAD = 4;   // row pitch of the transposition buffer: (HD/2+4)*2 bytes, i.e. 4 rows apart = 8 banks (mod 32)

template <int HD>
struct MfmaSmem {
    struct {
        uint32_t meta[WQ_WAVES][2][64];                  // per wave: K and V metadata words of the current block
        uint16_t vt[WQ_WAVES][32][HD / 2 + VT_PAD];      // per wave: half the channels of the V rows of a 16-bit block, read back transposed
    } run;
    // per-wave numerators for the merge; rows one bank apart.  A space of its own: a wavefront hands its numerators over
    // as soon as its loops end, while others still use the run-time part
    float O[WQ_WAVES][WQ_MAX_REP][HD + 1];
    U4 bq[4][HD / 32][64];                               // query operands of the four classes (index 3 = 16-bit segment), per lane
    float qx[4][2][64];                                  // ... with the head's power of two and the group's query sum
    float ml[WQ_WAVES][WQ_MAX_REP][2];
    unsigned next_ticket;                                // the workgroup's block counter
};


// ---- a lane's value next to that of lane ^ 16 and of lane ^ 32 -------------------------------------------------
// The row-swap instructions exchange rows of 16 lanes between two registers: given the same value x twice, the first
// register comes back holding the even row of every pair of rows in both of them (the lower half of the wavefront in
// both halves, for the 32-lane form), the second one the odd row (the upper half).  No LDS, no waiting.
struct RowPair { float even, odd; };
__device__ __forceinline__ RowPair rows_16(float x)
{
    const auto r = __builtin_amdgcn_permlane16_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    return RowPair{__uint_as_float(r[0]), __uint_as_float(r[1])};
}
__device__ __forceinline__ RowPair halves_32(float x)
{
    const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    return RowPair{__uint_as_float(r[0]), __uint_as_float(r[1])};
}
// sum / maximum over the four lanes {l, l ^ 16, l ^ 32, l ^ 48}, in every one of them
__device__ __forceinline__ float sum_over_rows(float x)
{
    const RowPair a = rows_16(x);
    const RowPair b = halves_32(a.even + a.odd);
    return b.even + b.odd;
}
__device__ __forceinline__ float max_over_rows(float x)
{
    const RowPair a = rows_16(x);
    const RowPair b = halves_32(fmaxf(a.even, a.odd));
    return fmaxf(b.even, b.odd);
}

// ---- the query operands of one class, built by the wavefront itself -------------------------------------------
// Lane (j, (g,h)) loads its quarter j of head h's query straight from global memory (hd/4 values), the head's
// largest magnitude is found with two cross-lane exchanges, the query is scaled by a power of two into [-1, 1)
// and laid out as the B operands of the k-steps: slot e of k-step r takes channel k_slot(c, r, e) of the quarter,
// times 2^-shift of that slot; lanes whose quarter is not in their column's group hold zeros (block-diagonal B).
// Returns the head's power of two (1 for the raw-bf16 operands of a bf16 16-bit segment) and the sum of the scaled
// query over the lane's group.
template <int HD, int CLS>
__device__ __forceinline__ void build_q_operands(const DecodeArgs& a, int b, int kvh, bool raw_bf16, U4* Bq, float& qexp, float& qsum)
{
    constexpr int QC = HD / 4, NK = HD / 32;
    const int lane = threadIdx.x & 63;
    const int j = lane >> 4, g = (lane & 15) >> 3, h = lane & 7;
    const bool live = h < a.rep;
    const int64_t base = ((int64_t)b * a.Hq + kvh * a.rep + (live ? h : 0)) * HD + j * QC;
    float v[QC];
    if (a.q_dtype == WQ_F32) {
        const float* p = static_cast<const float*>(a.q) + base;
#pragma unroll
        for (int k = 0; k < QC; k += 8) wq_ld8(p + k, v + k);
    } else if (a.q_dtype == WQ_BF16) {
        const __hip_bfloat16* p = static_cast<const __hip_bfloat16*>(a.q) + base;
#pragma unroll
        for (int k = 0; k < QC; k += 8) wq_ld8(p + k, v + k);
    } else {
        const __half* p = static_cast<const __half*>(a.q) + base;
#pragma unroll
        for (int k = 0; k < QC; k += 8) wq_ld8(p + k, v + k);
    }
    float mx = 0.f;
#pragma unroll
    for (int k = 0; k < QC; k++) mx = fmaxf(mx, fabsf(v[k]));   // (the columns of heads that do not exist repeat head 0: nobody reads them)
    mx = max_over_rows(mx);
    const int eb = (int)((__float_as_uint(mx) >> 23) & 0xFFu);              // biased exponent of the largest |q|
    const bool ok = eb > 0 && eb < 253;                                       // zero, denormal or non-finite: leave as is
    const float dn = ok ? __uint_as_float((uint32_t)(253 - eb) << 23) : 1.0f;     // 2^-(eb-126): max |q| lands in [0.5, 1)
    const float up = ok ? __uint_as_float((uint32_t)(eb + 1) << 23) : 1.0f;       // 2^(eb-126)
    float s = 0.f;                                 // sum of the scaled query as f16 holds it, two channels per instruction
#pragma unroll
    for (int k = 0; k < QC; k += 2) {
        const half2v pair_k = {(_Float16)(v[k] * dn), (_Float16)(v[k + 1] * dn)};
        s = __builtin_amdgcn_fdot2(pair_k, half2v{(_Float16)1.0f, (_Float16)1.0f}, s, false);
    }
    const RowPair quarters = rows_16(s);
    const float pair = quarters.even + quarters.odd;                         // both quarters of group j/2
    const RowPair groups = halves_32(pair);
    const float other = (lane & 32) ? groups.even : groups.odd;
    const bool mine = (j >> 1) == g;
    qsum = mine ? pair : other;
    qexp = raw_bf16 ? 1.0f : up;
#pragma unroll
    for (int r = 0; r < NK; r++) {
        uint32_t w[4];
#pragma unroll
        for (int e2 = 0; e2 < 4; e2++) {
            uint32_t half[2];
#pragma unroll
            for (int t = 0; t < 2; t++) {
                int ch, sh;
                k_slot(CLS, r, 2 * e2 + t, ch, sh);
                const _Float16 f = (_Float16)(v[ch] * dn * __uint_as_float((uint32_t)(127 - sh) << 23));
                half[t] = raw_bf16 ? (__float_as_uint(v[ch]) >> 16) : (uint32_t)__builtin_bit_cast(uint16_t, f);
            }
            w[e2] = mine ? (half[0] | (half[1] << 16)) : 0u;
        }
        Bq[r] = U4{w[0], w[1], w[2], w[3]};
    }
}

// The wavefronts of a workgroup walk the same classes, so the workgroup builds the operands of all four once, one
// class per wavefront (the first four), and keeps them in LDS.
template <int HD>
__device__ __forceinline__ void stage_q_operands(const DecodeArgs& a, MfmaSmem<HD>& sm, int b, int kvh, int wave, bool bf16seg)
{
    constexpr int NK = HD / 32;
    const int lane = threadIdx.x & 63;
    U4 Bq[NK];
    float qexp, qsum;
    if (wave >= 4) return;
    if (wave == 0) build_q_operands<HD, 0>(a, b, kvh, false, Bq, qexp, qsum);
    else if (wave == 1) build_q_operands<HD, 1>(a, b, kvh, false, Bq, qexp, qsum);
    else if (wave == 2) build_q_operands<HD, 2>(a, b, kvh, false, Bq, qexp, qsum);
    else build_q_operands<HD, 3>(a, b, kvh, bf16seg, Bq, qexp, qsum);
#pragma unroll
    for (int r = 0; r < NK; r++) sm.bq[wave][r][lane] = Bq[r];
    sm.qx[wave][0][lane] = qexp;
    sm.qx[wave][1][lane] = qsum;
}

template <int HD>
__device__ __forceinline__ void fetch_q_operands(const MfmaSmem<HD>& sm, int c, U4* Bq, float& qexp, float& qsum)
{
    const int lane = threadIdx.x & 63;
#pragma unroll
    for (int r = 0; r < HD / 32; r++) Bq[r] = sm.bq[c][r][lane];
    qexp = sm.qx[c][0][lane];
    qsum = sm.qx[c][1][lane];
}

// ---- shares of the token axis ---------------------------------------------------------------------------------
// A workgroup owns a contiguous cost range of the stream [16-bit | 8-bit | 4-bit | 2-bit] of its (sequence, KV
// head).  Its wavefronts do not run at the same speed (of the two that share a SIMD the older one gets more issue
// slots and more of the memory system, and the classes differ), and one that is done early cannot be replaced: the
// launch is over when the slowest wavefront is.  So the 32-token blocks of the range are handed out in stream
// order through a counter in LDS (a ticket = one block): whoever is free takes the next one.  A wavefront holds a
// range of tickets (normally one) and keeps tickets that stand for blocks of a later class until it gets there.
// The ticket that replaces a spent one is drawn at the start of a block's arithmetic and read at its end; LDS
// operations have a counter of their own, so the draw never waits for the block loads that are in flight.
// With WQ_DECODE_FIXED_SHARES the range is divided among the wavefronts by cost instead and no tickets are drawn.
struct Tickets {
    unsigned* ctr;      // the workgroup's counter (LDS)
    unsigned held, end; // tickets held: [held, end)
    bool spent;         // none left: another one is due
    bool synced;        // this wavefront has passed the workgroup's set-up barrier
    unsigned taper;     // from this ticket on (the workgroup's last WQ_TAPER_TICKETS) a wavefront refills only every other pipeline slot
};

// The set-up barrier (staged query operands, initial value of the block counter) is taken by every wavefront
// exactly once: after the first loads of the first class it walks have been issued, or, by a wavefront that has
// no blocks at all, before the final merge.
__device__ __forceinline__ void pass_setup_barrier(Tickets& t)
{
    if (!t.synced) {
        __syncthreads();
        t.synced = true;
    }
}

// lane 0 draws n tickets; the first one's value is valid in lane 0 once the LDS operation has returned
__device__ __forceinline__ unsigned draw_tickets(unsigned* ctr, unsigned n)
{
    unsigned v = 0;
    if ((threadIdx.x & 63) == 0) v = __hip_atomic_fetch_add(ctr, n, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
    return v;
}

__device__ __forceinline__ unsigned ticket_value(unsigned v) { return (unsigned)__builtin_amdgcn_readfirstlane((int)v); }

struct BlockSrc {
    int cur, end;            // this wavefront's own blocks of the class
    int pool_first;          // first block of the class's part of the workgroup's pool
    unsigned tk_lo, tk_hi;   // tickets that stand for those pool blocks
};

// draws n tickets and waits for them (filling the pipeline at the start of a class)
__device__ __forceinline__ void settle_tickets(Tickets& t, unsigned n)
{
    if (t.spent) {
        t.held = ticket_value(draw_tickets(t.ctr, n));
        t.end = t.held + n;
        t.spent = false;
    }
}

__device__ __forceinline__ bool has_blocks(const BlockSrc& s, Tickets& t, unsigned fill)
{
    if (s.cur < s.end) return true;
    if (s.tk_lo >= s.tk_hi) return false;
    settle_tickets(t, fill);
    return t.held < s.tk_hi;
}

// next block of the class for this wavefront, or -1 (and then -1 on every later call for the class)
__device__ __forceinline__ int next_block(BlockSrc& s, Tickets& t, unsigned fill)
{
    if (s.cur < s.end) return s.cur++;
    if (s.tk_lo >= s.tk_hi) return -1;
    settle_tickets(t, fill);
    if (t.held >= s.tk_hi) return -1;        // a block of a later class, or none: keep the tickets
    const unsigned v = t.held++;
    t.spent = t.held == t.end;
    return s.pool_first + (int)(v - s.tk_lo);
}

template <int HD, int BITS>
struct Frag {
    static constexpr int KDW = (HD / 4) * BITS / 32;        // dwords of K codes per lane per 16-token tile
    static constexpr int VDW = (HD / 16) * 8 * BITS / 32;   // dwords of V codes per lane per 32-token block
    uint32_t k[2][KDW];
    uint32_t v[VDW];
    uint32_t km, vm;                                        // one metadata word per lane and plane
};

template <int N>
__device__ __forceinline__ void load_dwords(const uint32_t* __restrict__ p, uint32_t* dst)
{
    if constexpr (N == 1) {
        dst[0] = p[0];
    } else if constexpr (N == 2) {
        uint2 u = *reinterpret_cast<const uint2*>(p);
        dst[0] = u.x;
        dst[1] = u.y;
    } else {
#pragma unroll
        for (int d = 0; d < N; d += 4) {
            uint4 u = *reinterpret_cast<const uint4*>(p + d);
            dst[d] = u.x;
            dst[d + 1] = u.y;
            dst[d + 2] = u.z;
            dst[d + 3] = u.w;
        }
    }
}

// One class of one (sequence, KV head): this wavefront's share of its 32-token blocks (len tokens from token slot
// tok_base of the class buffers).
template <int HD, int BITS, int DEPTH>
__device__ __forceinline__ void walk_class_mfma(const DecodeArgs& a, MfmaSmem<HD>& sm, int b, int kvh, int len, int tok_base, BlockSrc& src,
                                                Tickets& tk, float c_log2, WaveState<HD>& st)
{
    constexpr int C = BITS == 2 ? 0 : (BITS == 4 ? 1 : 2);
    constexpr int NK = HD / 32;                    // k-steps of the logit product per 16-token tile
    constexpr int CT = HD / 16;                    // channel tiles of the value product
    using F = Frag<HD, BITS>;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int j = lane >> 4, col = lane & 15, g = col >> 3;

    if (!has_blocks(src, tk, DEPTH)) return;
    const wq_packed_kv& kv = a.kv;
    const int64_t cap = kv.cap[C];
    const uint8_t* kbase = static_cast<const uint8_t*>(kv.codes[C]) + ((int64_t)kvh * cap + tok_base) * HD * BITS / 8 + lane * (F::KDW * 4);
    const uint8_t* vbase = static_cast<const uint8_t*>(kv.codes[C]) + (((int64_t)kv.Hkv + kvh) * cap + tok_base) * HD * BITS / 8 + lane * (F::VDW * 4);
    const uint32_t* kmeta = static_cast<const uint32_t*>(kv.meta[C]) + ((int64_t)kvh * cap + tok_base) * 2 + lane;
    const uint32_t* vmeta = static_cast<const uint32_t*>(kv.meta[C]) + (((int64_t)kv.Hkv + kvh) * cap + tok_base) * 2 + lane;
    uint32_t* smeta = &sm.run.meta[wave][0][0];
    const int moff = g * 16 + 4 * j;               // (group g, tokens 4j..4j+3) inside a metadata tile of 32 words

    auto load = [&](int blk, F& f) {
        const int64_t o = (int64_t)blk * (32 * HD * BITS / 8);
        load_dwords<F::KDW>(reinterpret_cast<const uint32_t*>(kbase + o), f.k[0]);
        load_dwords<F::KDW>(reinterpret_cast<const uint32_t*>(kbase + o + 16 * HD * BITS / 8), f.k[1]);
        load_dwords<F::VDW>(reinterpret_cast<const uint32_t*>(vbase + o), f.v);
        f.km = kmeta[(int64_t)blk * 64];
        f.vm = vmeta[(int64_t)blk * 64];
    };

    // software pipeline: DEPTH blocks in flight per wavefront; the first loads go out before anything else
    F f[DEPTH];
    int bi[DEPTH];
#pragma unroll
    for (int d = 0; d < DEPTH; d++) {
        bi[d] = next_block(src, tk, DEPTH - d);
        if (bi[d] >= 0) load(bi[d], f[d]);
    }
    pass_setup_barrier(tk);
    U4 Bqw[NK];
    float qexp, qsum;
    fetch_q_operands<HD>(sm, C, Bqw, qexp, qsum);
    half8 Bq[NK];
#pragma unroll
    for (int r = 0; r < NK; r++) Bq[r] = __builtin_bit_cast(half8, Bqw[r]);
    // logits come out of the matrix cores as 2^-24 * sum q' code; fold 2^24, the head's power of two and
    // sm_scale*log2(e) into one constant, and pre-divide the m-term by 2^24 so both terms share it.
    const float cexp = c_log2 * qexp * 16777216.0f;
    const float qs = qsum * (1.0f / 16777216.0f);

    // added to the logits: zero, except for the tokens past the end of the sequence's last block of the class
    // (the last block this wavefront gets: shares and tickets go up the stream), which get -inf
    float pen[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    // partial sums per slot register v: its weights carry 2^-shift(v) (folded into the exponent), undone after the loop
    float lv[4] = {0.f, 0.f, 0.f, 0.f}, av[4] = {0.f, 0.f, 0.f, 0.f}, ms[4];
#pragma unroll
    for (int v = 0; v < 4; v++) ms[v] = st.m + v_slot_shift<BITS>(v) - st.up;

    auto compute = [&](int blk, const F& f) {
        const bool redraw = tk.spent;
        unsigned drawn = 0;
        if (redraw) drawn = draw_tickets(tk.ctr, 1u);
        if (blk * 32 + 32 > len) {
            const int nv = len - blk * 32;         // valid tokens in this block
#pragma unroll
            for (int t = 0; t < 2; t++)
#pragma unroll
                for (int i = 0; i < 4; i++) pen[4 * t + i] = (16 * t + 4 * j + i >= nv) ? -INFINITY : 0.f;
        }
        // ---- scales and minima: one word per lane in, the lane's 4 tokens x 2 tiles x {K,V} out ----
        smeta[lane] = f.km;
        smeta[64 + lane] = f.vm;
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        uint32_t kw[8], vw[8];
#pragma unroll
        for (int t = 0; t < 2; t++) {
            const uint4 a = *reinterpret_cast<const uint4*>(smeta + t * 32 + moff);
            const uint4 c = *reinterpret_cast<const uint4*>(smeta + 64 + t * 32 + moff);
            kw[4 * t] = a.x, kw[4 * t + 1] = a.y, kw[4 * t + 2] = a.z, kw[4 * t + 3] = a.w;
            vw[4 * t] = c.x, vw[4 * t + 1] = c.y, vw[4 * t + 2] = c.z, vw[4 * t + 3] = c.w;
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();   // the next block's words may overwrite the buffer after this point

        // ---- logits of the two 16-token tiles ----
        float x[8];
#pragma unroll
        for (int t = 0; t < 2; t++) {
            floatx4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int r = 0; r < NK; r++) acc = mfma(k_operand<BITS>(f.k[t], r), Bq[r], acc);
#pragma unroll
            for (int i = 0; i < 4; i++) {
                const float y = fmaf(f16lo(kw[4 * t + i]), acc[i], fmaf(f16hi(kw[4 * t + i]), qs, pen[4 * t + i]));
                x[4 * t + i] = y + ror8(y);
            }
        }
        // ---- reference exponent: touch the other lane groups only when some logit is far above it ----
        float lm = max3(max3(x[0], x[1], x[2]), max3(x[3], x[4], x[5]), max3(x[6], x[7], x[7]));
        lm *= cexp;                                // cexp > 0
        if (__builtin_amdgcn_ballot_w64(lm > st.m + WQ_MAX_SLACK) != 0) {
            lm = max_over_rows(lm);
            const float mn = fmaxf(st.m, lm);
            const float alpha = (mn == -INFINITY) ? 1.0f : __builtin_amdgcn_exp2f(st.m - mn);   // 0 on the first block
            st.m = mn;
            st.l *= alpha;
            st.accM *= alpha;
#pragma unroll
            for (int v = 0; v < 4; v++) {
                lv[v] *= alpha;
                av[v] *= alpha;
                ms[v] = mn + v_slot_shift<BITS>(v) - st.up;
            }
#pragma unroll
            for (int ct = 0; ct < CT; ct++) st.O[ct] *= alpha;
        }
        // ---- weights with the slot's power of two folded into the exponent, P' = p * s_v, and the m_v part ----
        float p[8];
#pragma unroll
        for (int k = 0; k < 8; k++) {
            p[k] = __builtin_amdgcn_exp2f(fmaf(x[k], cexp, -ms[k & 3]));
            lv[k & 3] += p[k];
            av[k & 3] = fmaf(f16hi(vw[k]), p[k], av[k & 3]);
        }
        uint32_t bp[4];
#pragma unroll
        for (int v = 0; v < 4; v++)                // slots (2v, 2v+1) = (tile 0, tile 1) token 4j+v
            bp[v] = mul_f16lo_to_hi(mul_f16lo_to_lo(vw[v], p[v]), vw[4 + v], p[4 + v]);
        const half8 Bp = as_half8(bp[0], bp[1], bp[2], bp[3]);
        // ---- values ----
#pragma unroll
        for (int ct = 0; ct < CT; ct++) st.O[ct] = mfma(v_operand<BITS>(f.v, ct), Bp, st.O[ct]);
        const unsigned got = ticket_value(drawn);      // read on every path: nothing is left pending at the loop edge
        if (redraw) {
            tk.held = got;
            tk.end = got + 1u;
            tk.spent = false;
        }
    };

    while (bi[0] >= 0) {
#pragma unroll
        for (int d = 0; d < DEPTH; d++) {
            if (bi[d] >= 0) {
                compute(bi[d], f[d]);
                // near the end of the workgroup's range the odd slots are given up: whatever is in flight when the last
                // block has been handed out is arithmetic that no load overlaps with any more
                if ((d & 1) && DEPTH > 2 && tk.held >= tk.taper) {
                    bi[d] = -1;
                    continue;
                }
                bi[d] = next_block(src, tk, 1u);
                if (bi[d] >= 0) load(bi[d], f[d]);
            }
        }
    }
    const float down = pow2_of(-st.up);            // undoes the factor that the weights were formed with
#pragma unroll
    for (int v = 0; v < 4; v++) {
        st.l = fmaf(lv[v], down * (1.0f / v_slot_scale<BITS>(v)), st.l);
        st.accM = fmaf(av[v], down * (1.0f / v_slot_scale<BITS>(v)), st.accM);
    }
}

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

template <bool BF>
__device__ __forceinline__ floatx4 mfma16(uint32_t a0, uint32_t a1, uint32_t a2, uint32_t a3, const U4& b, floatx4 c)
{
    U4 a{a0, a1, a2, a3};
    if constexpr (BF)
        return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
    else
        return __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(half8, a), __builtin_bit_cast(half8, b), c, 0, 0, 0);
}

// The 16-bit segment (text, generated tokens, video tail, 16-bit windows) of one (sequence, KV head): rows are
// plain [token][Hkv][hd] so the K side feeds the matrix cores straight from global memory (one token row
// quarter per lane); V rows go through LDS and are read back one channel x 8 tokens per lane.  bf16 caches use
// the bf16 instruction with the exact bf16 query and the weights split into two bf16 terms (p = hi + lo);
// fp16 caches use the f16 instruction.  Accumulators are in true units here (no 2^-24).
template <int HD, bool BF>
// new_row >= 0: row new_row (= len - 1) is not in the cache yet: it is read from knew / vnew, this (sequence, KV head)'s
// [hd] slices of the token that the launch appends.
__device__ __forceinline__ void walk_seg16_mfma(const DecodeArgs& a, MfmaSmem<HD>& sm, int b, int kvh, int len, int first_row, BlockSrc& src,
                                                Tickets& tk, float c_log2, WaveState<HD>& st, int new_row, const uint16_t* knew,
                                                const uint16_t* vnew)
{
    constexpr int NK = HD / 32, CT = HD / 16, PITCH = HD / 2 + VT_PAD, KDW = HD / 8;
    if (!has_blocks(src, tk, 1u)) return;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int j = lane >> 4, col = lane & 15;
    const wq_packed_kv& kv = a.kv;
    const int64_t row0 = first_row;
    const int64_t rstride = (int64_t)kv.Hkv * HD;
    const uint16_t* k16 = static_cast<const uint16_t*>(kv.k16) + (int64_t)kvh * HD;
    const uint16_t* v16 = static_cast<const uint16_t*>(kv.v16) + (int64_t)kvh * HD;
    pass_setup_barrier(tk);
    U4 Bq[NK];
    float qexp, qsum;
    fetch_q_operands<HD>(sm, 3, Bq, qexp, qsum);
    const float cexp = c_log2 * qexp;
    uint16_t* vt = &sm.run.vt[wave][0][0];

    for (int blk = next_block(src, tk, 1u); blk >= 0; blk = next_block(src, tk, 1u)) {
        const int nv = len - blk * 32;
        const bool redraw = tk.spent;
        unsigned drawn = 0;
        if (redraw) drawn = draw_tickets(tk.ctr, 1u);
        // ---- all loads of the block up front: one memory round trip per block ----
        uint32_t kd[2][KDW];
#pragma unroll
        for (int t = 0; t < 2; t++) {
            const int tok = min(blk * 32 + 16 * t + col, len - 1);      // rows past the end re-read the last row, masked below
            const uint16_t* src_k = tok == new_row ? knew : k16 + (row0 + tok) * rstride;
            load_dwords<KDW>(reinterpret_cast<const uint32_t*>(src_k + j * (HD / 4)), kd[t]);
        }
        constexpr int VIT = (32 * (HD / 2) * 2) / (16 * 64);          // 16-byte pieces per lane and channel half
        uint4 vd[2][VIT];
#pragma unroll
        for (int half = 0; half < 2; half++)
#pragma unroll
            for (int it = 0; it < VIT; it++) {
                const int chunk = it * 64 + lane;
                const int row = chunk / (HD / 16), c16 = chunk % (HD / 16);
                const int tok = min(blk * 32 + row, len - 1);
                const uint16_t* src_v = tok == new_row ? vnew : v16 + (row0 + tok) * rstride;
                vd[half][it] = *reinterpret_cast<const uint4*>(src_v + half * (HD / 2) + c16 * 8);
            }
        // ---- logits ----
        float x[8];
#pragma unroll
        for (int t = 0; t < 2; t++) {
            floatx4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int r = 0; r < NK; r++) acc = mfma16<BF>(kd[t][4 * r], kd[t][4 * r + 1], kd[t][4 * r + 2], kd[t][4 * r + 3], Bq[r], acc);
#pragma unroll
            for (int i = 0; i < 4; i++) x[4 * t + i] = acc[i] + ror8(acc[i]);
        }
        if (nv < 32) {
#pragma unroll
            for (int t = 0; t < 2; t++)
#pragma unroll
                for (int i = 0; i < 4; i++)
                    if (16 * t + 4 * j + i >= nv) x[4 * t + i] = -INFINITY;
        }
        float lm = fmaxf(fmaxf(fmaxf(x[0], x[1]), fmaxf(x[2], x[3])), fmaxf(fmaxf(x[4], x[5]), fmaxf(x[6], x[7])));
        lm *= cexp;
        if (__builtin_amdgcn_ballot_w64(lm > st.m + WQ_MAX_SLACK) != 0) {
            lm = max_over_rows(lm);
            const float mn = fmaxf(st.m, lm);
            const float alpha = (mn == -INFINITY) ? 1.0f : __builtin_amdgcn_exp2f(st.m - mn);
            st.m = mn;
            st.l *= alpha;
            st.accM *= alpha;
#pragma unroll
            for (int ct = 0; ct < CT; ct++) st.O[ct] *= alpha;
        }
        float p[8];
#pragma unroll
        for (int k = 0; k < 8; k++) {
            p[k] = __builtin_amdgcn_exp2f(fmaf(x[k], cexp, -st.m));
            st.l += p[k];
        }
        // ---- weights as B operands: slots (2v, 2v+1) = (tile 0 token 4j+v, tile 1 token 4j+v) ----
        U4 Ph, Pl;
        {
            uint32_t hi[4], lo[4];
#pragma unroll
            for (int v = 0; v < 4; v++) {
                if constexpr (BF) {
                    const uint32_t u0 = __float_as_uint(p[v]), u1 = __float_as_uint(p[4 + v]);
                    const float r0 = p[v] - __uint_as_float(u0 & 0xFFFF0000u), r1 = p[4 + v] - __uint_as_float(u1 & 0xFFFF0000u);
                    hi[v] = (u0 >> 16) | (u1 & 0xFFFF0000u);
                    lo[v] = (__float_as_uint(r0) >> 16) | (__float_as_uint(r1) & 0xFFFF0000u);
                } else {
                    const _Float16 h0 = (_Float16)p[v], h1 = (_Float16)p[4 + v];
                    hi[v] = (uint32_t)__builtin_bit_cast(uint16_t, h0) | ((uint32_t)__builtin_bit_cast(uint16_t, h1) << 16);
                    lo[v] = 0;
                }
            }
            Ph = U4{hi[0], hi[1], hi[2], hi[3]};
            Pl = U4{lo[0], lo[1], lo[2], lo[3]};
        }
        // ---- V rows -> LDS -> one channel x 8 tokens per lane, half of the channels at a time ----
#pragma unroll
        for (int half = 0; half < 2; half++) {
#pragma unroll
            for (int it = 0; it < VIT; it++) {
                const int chunk = it * 64 + lane;
                const int row = chunk / (HD / 16), c16 = chunk % (HD / 16);
                const uint4 v = vd[half][it];
                uint2* dst = reinterpret_cast<uint2*>(vt + row * PITCH + c16 * 8);   // the padded pitch is only 8-byte aligned
                dst[0] = uint2{v.x, v.y};
                dst[1] = uint2{v.z, v.w};
            }
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
#pragma unroll
            for (int c2 = 0; c2 < CT / 2; c2++) {
                const int ct = half * (CT / 2) + c2;
                uint32_t a[4];
#pragma unroll
                for (int v = 0; v < 4; v++) {
                    const uint32_t e0 = vt[(4 * j + v) * PITCH + 16 * c2 + col];
                    const uint32_t e1 = vt[(16 + 4 * j + v) * PITCH + 16 * c2 + col];
                    a[v] = e0 | (e1 << 16);
                }
                st.O[ct] = mfma16<BF>(a[0], a[1], a[2], a[3], Ph, st.O[ct]);
                if constexpr (BF) st.O[ct] = mfma16<BF>(a[0], a[1], a[2], a[3], Pl, st.O[ct]);
            }
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();          // the buffer is overwritten next
        }
        const unsigned got = ticket_value(drawn);
        if (redraw) {
            tk.held = got;
            tk.end = got + 1u;
            tk.spent = false;
        }
    }
}

// ---- a launch that appends a token (k_new != NULL) must not change len16[b] while a workgroup of sequence b may still
// read it (under WQ_DECODE_BY_LENGTH the split count of a sequence depends on its length).  Every workgroup of the
// sequence, also one that has nothing to do, counts itself on the sequence's counter once the tables are in its registers
// (an add that returns nothing: nobody waits for it).  The sequence's last workgroup in dispatch order (highest KV head,
// highest split; every other one of the sequence was dispatched before it and waits for nobody before it counts itself)
// waits at its very end until the count is complete, clears the counter for the next launch and writes the new length.
constexpr long long WQ_APPEND_WAIT_TICKS = 400000000ll;   // 4 s of the 100 MHz clock: far beyond any launch; a wait that long gives up

__device__ __forceinline__ void note_tables_read(const DecodeArgs& a, int b, int len16_read)
{
    if (a.k_new && threadIdx.x == 0) {
        unsigned one = 1u;
        asm volatile("; the count follows the read of len16 %1" : "+s"(one) : "s"(len16_read));
        __hip_atomic_fetch_add(a.arrive + (a.B * a.kv.Hkv + b) * WQ_ARRIVE_STRIDE, one, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
}

__device__ __forceinline__ void finish_append(const DecodeArgs& a, int b, int kvh, int split, int new_row)
{
    if (!a.k_new || threadIdx.x != 0 || kvh != a.kv.Hkv - 1 || split != a.splits - 1) return;
    unsigned* ctr = a.arrive + (a.B * a.kv.Hkv + b) * WQ_ARRIVE_STRIDE;
    const unsigned all = (unsigned)a.kv.Hkv * (unsigned)a.splits;
    const long long t_start = wall_clock64();
    while (__hip_atomic_load(ctr, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != all) {
        if (wall_clock64() - t_start > WQ_APPEND_WAIT_TICKS) {
            atomicOr(a.status, WQ_DEV_APPEND_TIMEOUT);
            break;
        }
        __builtin_amdgcn_s_sleep(8);
    }
    __hip_atomic_store(ctr, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    if (new_row >= 0) a.kv.len16[b] = new_row + 1;
}

// Shares are laid out on a cost axis in integers (a 32-token block of a class costs WQ_BLOCK_COST of it): everything
// here depends only on the sequence's tables and the workgroup's and wavefront's numbers, which are the same for all
// lanes, so the compiler keeps it in scalar registers and on the scalar unit, where it does not compete with the vector
// work of the wavefront that shares the SIMD (as float arithmetic on the vector unit it held every wavefront's first
// loads back by most of a microsecond).  Every wavefront evaluates the same expressions for the same boundary, so
// neighbouring shares meet exactly, and the mapping is monotone, which is all that the partition needs.
// first block of a class (n blocks of cost W each, starting at cost `base`) at or after cost x
template <unsigned W>
__device__ __forceinline__ int range_edge(unsigned x, unsigned base, int n)
{
    const unsigned e = x > base ? (x - base + (W - 1u)) / W : 0u;             // (division by a constant: a multiplication)
    return (int)min(e, (unsigned)n);
}

__device__ __forceinline__ int range_edge_of(int c, unsigned x, unsigned base, int n)
{
    return c == 0 ? range_edge<(unsigned)WQ_BLOCK_COST[0]>(x, base, n)
         : c == 1 ? range_edge<(unsigned)WQ_BLOCK_COST[1]>(x, base, n)
         : c == 2 ? range_edge<(unsigned)WQ_BLOCK_COST[2]>(x, base, n)
                  : range_edge<(unsigned)WQ_BLOCK_COST[3]>(x, base, n);
}

// ---- helpers of the two merges --------------------------------------------------------------------------------
typedef float floatx2 __attribute__((ext_vector_type(2)));
template <int N> struct FloatN;
template <> struct FloatN<1> { typedef float type; };
template <> struct FloatN<2> { typedef floatx2 type; };
template <int N> __device__ __forceinline__ float part_elem(typename FloatN<N>::type v, int c);
template <> __device__ __forceinline__ float part_elem<1>(float v, int) { return v; }
template <> __device__ __forceinline__ float part_elem<2>(floatx2 v, int c) { return v[c]; }

// N floats (N * 4 bytes, aligned to that) to memory with a device-scope store (one instruction)
template <int N>
__device__ __forceinline__ void store_through(float* p, const float* v)
{
    if constexpr (N == 1) {
        __hip_atomic_store(p, v[0], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    } else {
        static_assert(N == 2, "one or two floats");
        const unsigned long long u = (unsigned long long)__float_as_uint(v[0]) | ((unsigned long long)__float_as_uint(v[1]) << 32);
        __hip_atomic_store(reinterpret_cast<unsigned long long*>(p), u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
}

template <int N>
__device__ __forceinline__ void store_plain(float* p, const float* v)
{
    if constexpr (N == 1) {
        p[0] = v[0];
    } else {
        static_assert(N == 2, "one or two floats");
        *reinterpret_cast<float2*>(p) = make_float2(v[0], v[1]);
    }
}

// N floats of a partial through a buffer descriptor, with a device-scope load (does not stop at a cache); zero
// when the offset is beyond the descriptor's range
template <int N>
__device__ __forceinline__ typename FloatN<N>::type ld_part(__amdgpu_buffer_rsrc_t rsrc, unsigned byte_off)
{
    constexpr int DEVICE_SCOPE = 16;               // the sc1 bit of the instruction
    if constexpr (N == 1) {
        return __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(rsrc, (int)byte_off, 0, DEVICE_SCOPE));
    } else {
        static_assert(N == 2, "one or two floats");
        return __builtin_bit_cast(floatx2, __builtin_amdgcn_raw_buffer_load_b64(rsrc, (int)byte_off, 0, DEVICE_SCOPE));
    }
}


template <int HD>
__device__ void wq_decode_mfma_body(const DecodeArgs& a, void* smem_raw)
{
    MfmaSmem<HD>& sm = *reinterpret_cast<MfmaSmem<HD>*>(smem_raw);
    // consecutive workgroups go to different (sequence, KV head) units: the units' tables and queries are then
    // read by all XCDs alike, and the workgroups of one unit do not start in a burst on neighbouring compute units
    // (the grid is (KV heads, sequences, splits): workgroups are dispatched with x fastest, and nothing here has to divide)
    const int kvh = (int)blockIdx.x, b = (int)blockIdx.y, split = (int)blockIdx.z;
    const int unit = b * a.kv.Hkv + kvh;
    const int tid = threadIdx.x, wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63;
    const int j = lane >> 4, col = lane & 15, g = col >> 3, h = col & 7;
    constexpr int CT = HD / 16;
    const bool bf16seg = a.kv.dtype16 == WQ_BF16;
    WQ_STAMP(0);

    // ---- the sequence's tables first (their loads are in flight while the query operands are built) ----
    int cls_len[4], cls_off[4];
#pragma unroll
    for (int c = 0; c < 3; c++) {
        cls_len[c] = a.kv.cls_len[c][b];
        cls_off[c] = a.kv.cls_off[c][b];
    }
    cls_len[3] = a.kv.len16[b];
    cls_off[3] = a.kv.off16[b];
    const float v_scale_max = a.kv.v_scale_max[b];
    note_tables_read(a, b, cls_len[3]);
    // a token appended by this launch becomes the last row of the 16-bit segment: read from k_new / v_new by whoever
    // walks its block, copied into the cache by the first split's workgroup, counted in len16 once every workgroup of
    // the sequence has read len16 (finish_append)
    int new_row = -1;
    const uint16_t *knew = nullptr, *vnew = nullptr;
    if (a.k_new) {
        const int64_t row = (int64_t)cls_off[3] + cls_len[3];
        if (row < a.kv.off16[b + 1] && row < a.kv.cap16) {
            new_row = cls_len[3];
            cls_len[3] += 1;
            knew = a.k_new + ((int64_t)b * a.kv.Hkv + kvh) * HD;
            vnew = a.v_new + ((int64_t)b * a.kv.Hkv + kvh) * HD;
            if (split == 0 && tid < 2 * (HD / 8)) {
                const int plane = tid / (HD / 8), piece = tid % (HD / 8);
                uint16_t* dst = static_cast<uint16_t*>(plane ? a.kv.v16 : a.kv.k16) + (row * a.kv.Hkv + kvh) * HD + piece * 8;
                *reinterpret_cast<uint4*>(dst) = *reinterpret_cast<const uint4*>((plane ? vnew : knew) + piece * 8);
            }
        } else if (split == 0 && kvh == 0 && tid == 0) {
            atomicOr(a.status, WQ_DEV_SEG16_OVERFLOW);      // the segment is full: nothing is appended
        }
    }
    WQ_WSTAMP(5, wall_clock64() + (long long)((cls_len[0] + cls_len[1] + cls_len[2] + cls_len[3] + cls_off[0] + cls_off[1] + cls_off[2] + cls_off[3]) & 0));   // the tables have arrived
    // ---- splits of this (sequence, KV head): all of the launch's, or, in a launch for sequences of different lengths,
    //      as many as the sequence's share of the longest one asks for; the workgroups beyond them have nothing to do ----
    int S = a.splits;
    if (a.len_scale > 0.f) {
        const int tokens = cls_len[0] + cls_len[1] + cls_len[2] + cls_len[3];
        S = max(1, min(a.splits, (int)ceilf((float)tokens * a.len_scale)));
        if (split >= S) {
            finish_append(a, b, kvh, split, new_row);
            return;
        }
    }
    if (tid == 0) sm.next_ticket = (unsigned)(WQ_FIRST_TICKETS * WQ_WAVES);
    // ---- the query operands of all classes, one class per wavefront ----
    stage_q_operands<HD>(a, sm, b, kvh, wave, bf16seg);

    // ---- the workgroup's range of the stream [16-bit | 8-bit | 4-bit | 2-bit] of (b, kvh), and this wavefront's
    //      fixed share of it (none unless the launch asks for fixed shares: then there is no pool) ----
    Tickets tk;
    tk.ctr = &sm.next_ticket;
    // the first tickets are fixed (WQ_FIRST_TICKETS consecutive blocks per wavefront), so that the first loads can go
    // out before the workgroup's set-up barrier; the counter starts behind them
    tk.held = (unsigned)(wave * WQ_FIRST_TICKETS);
    tk.end = tk.held + (unsigned)WQ_FIRST_TICKETS;
    tk.spent = false;
    tk.synced = false;
    tk.taper = 0xFFFFFFFFu;
    BlockSrc src[4];
    {
        int nb[4];
#pragma unroll
        for (int c = 0; c < 3; c++) nb[c] = (cls_len[c] + 31) >> 5;
        nb[3] = a.mfma16 ? (cls_len[3] + 31) >> 5 : 0;
        unsigned total = 0u;
#pragma unroll
        for (int c = 0; c < 4; c++) total += (unsigned)nb[c] * (unsigned)WQ_BLOCK_COST[c];
        // cost at which split x starts: floor(total * x / S) up to rounding (one reciprocal, the same bits in every
        // wavefront of the launch); split 0 starts at cost 0, the last one ends behind everything
        const float rS = __builtin_amdgcn_rcpf((float)S);
        auto start_of = [&](int x) {
            return min(total, (unsigned)__builtin_amdgcn_readfirstlane((int)(unsigned)((float)total * ((float)x * rS))));
        };
        const unsigned G0 = split == 0 ? 0u : start_of(split);
        const unsigned G1 = split == S - 1 ? total : start_of(split + 1);
        unsigned base = 0u;
        unsigned t = 0;
#pragma unroll
        for (int c = 3; c >= 0; c--) {
            const int e0 = range_edge_of(c, G0, base, nb[c]);
            const int e1 = range_edge_of(c, G1, base, nb[c]);
            if (a.fixed_shares) {                  // the range is divided among the wavefronts by cost; no pool
                const unsigned long long span = G1 - G0;
                const unsigned x0 = G0 + (unsigned)((span * (unsigned)wave) >> 3), x1 = G0 + (unsigned)((span * (unsigned)(wave + 1)) >> 3);
                static_assert(WQ_WAVES == 8, "the shift above");
                src[c].cur = wave == 0 ? e0 : range_edge_of(c, x0, base, nb[c]);
                src[c].end = wave == WQ_WAVES - 1 ? e1 : range_edge_of(c, x1, base, nb[c]);
                src[c].pool_first = e1;
                src[c].tk_lo = src[c].tk_hi = t;
            } else {                               // the whole range is the pool
                src[c].cur = src[c].end = 0;
                src[c].pool_first = e0;
                src[c].tk_lo = t;
                t += (unsigned)(e1 - e0);
                src[c].tk_hi = t;
            }
            base += (unsigned)nb[c] * (unsigned)WQ_BLOCK_COST[c];
        }
        if (!a.fixed_shares && t > (unsigned)WQ_TAPER_TICKETS) tk.taper = t - (unsigned)WQ_TAPER_TICKETS;
    }

    WQ_STAMP(1);
#ifdef WQ_TIMELINE
    if (a.dbg && threadIdx.x == 0) {
        a.dbg[WQ_WG * 64 + 6] = __builtin_amdgcn_s_getreg((31 << 11) | 4);    // HW_ID
        a.dbg[WQ_WG * 64 + 7] = -(long long)__builtin_readcyclecounter();
    }
#endif

    WaveState<HD> st;
#pragma unroll
    for (int ct = 0; ct < CT; ct++) st.O[ct] = floatx4{0.f, 0.f, 0.f, 0.f};
    st.m = -INFINITY;
    st.l = 0.f;
    st.accM = 0.f;
    st.up = weight_upscale(v_scale_max);
    const float o_unit = pow2_of(24.0f - st.up);   // what an accumulator of the value product counts in units of
    const float c_log2 = a.sm_scale * 1.4426950408889634f;
    WQ_WSTAMP(0, wall_clock64());
    if (has_blocks(src[3], tk, 1u)) {              // (most wavefronts have no block of the 16-bit segment and go straight on)
        if (bf16seg)
            walk_seg16_mfma<HD, true>(a, sm, b, kvh, cls_len[3], cls_off[3], src[3], tk, c_log2, st, new_row, knew, vnew);
        else
            walk_seg16_mfma<HD, false>(a, sm, b, kvh, cls_len[3], cls_off[3], src[3], tk, c_log2, st, new_row, knew, vnew);
        // the quantized classes accumulate 2^(up-24) * (p s_v code); bring the 16-bit part to the same unit (exact)
        const float to_unit = pow2_of(st.up - 24.0f);
#pragma unroll
        for (int ct = 0; ct < CT; ct++) st.O[ct] *= to_unit;
    }
    WQ_WSTAMP(1, wall_clock64());
    walk_class_mfma<HD, 8, WQ_D8>(a, sm, b, kvh, cls_len[2], cls_off[2], src[2], tk, c_log2, st);
    WQ_WSTAMP(2, wall_clock64());
    walk_class_mfma<HD, 4, WQ_D4>(a, sm, b, kvh, cls_len[1], cls_off[1], src[1], tk, c_log2, st);
    WQ_WSTAMP(3, wall_clock64());
    walk_class_mfma<HD, 2, WQ_D2>(a, sm, b, kvh, cls_len[0], cls_off[0], src[0], tk, c_log2, st);
    WQ_WSTAMP(4, wall_clock64());

    WQ_STAMP(4);
#ifdef WQ_TIMELINE
    if (a.dbg && threadIdx.x == 0) a.dbg[WQ_WG * 64 + 7] += (long long)__builtin_readcyclecounter();
#endif
    // ---- reduce the lane groups' shares, hand the wave's numerators to LDS ----
    float l = st.l, am = st.accM;
    l = sum_over_rows(l);
    am = sum_over_rows(am);
#pragma unroll
    for (int ct = 0; ct < CT; ct++) {
        if ((ct >= CT / 2) == (g == 1)) {          // this column's group owns channel tile ct
#pragma unroll
            for (int i = 0; i < 4; i++) sm.O[wave][h][16 * ct + 4 * j + i] = fmaf(st.O[ct][i], o_unit, am);
        }
    }
    if (j == 0 && g == 0) {
        sm.ml[wave][h][0] = st.m;
        sm.ml[wave][h][1] = l;
    }
    pass_setup_barrier(tk);
    __syncthreads();
    // ---- merge the wavefronts, write the partial (m in natural-log units): wavefront r takes head r, a lane CPL
    //      neighbouring channels, so the eight scales of a head are computed once per lane ----
    constexpr int CPL = HD / 64;                   // channels per lane
    static_assert(WQ_WAVES >= WQ_MAX_REP, "one wavefront per head");
    const int64_t pstride = (int64_t)a.rep * (HD + 2);
    float* pbase = a.part + ((int64_t)unit * a.nparts) * pstride;
    if (wave < a.rep) {
        float* out = pbase + split * pstride + wave * (HD + 2);
        float mw[WQ_WAVES];
#pragma unroll
        for (int w = 0; w < WQ_WAVES; w++) mw[w] = sm.ml[w][wave][0];
        float M = mw[0];
#pragma unroll
        for (int w = 1; w < WQ_WAVES; w++) M = fmaxf(M, mw[w]);
        float num[CPL], L = 0.f;
#pragma unroll
        for (int c = 0; c < CPL; c++) num[c] = 0.f;
#pragma unroll
        for (int w = 0; w < WQ_WAVES; w++) {
            const float sc = (mw[w] == -INFINITY) ? 0.f : __builtin_amdgcn_exp2f(mw[w] - M);
#pragma unroll
            for (int c = 0; c < CPL; c++) num[c] = fmaf(sm.O[w][wave][CPL * lane + c], sc, num[c]);
            L = fmaf(sm.ml[w][wave][1], sc, L);
        }
        // device-scope stores go through to memory (every XCD has an L2 of its own), so that no cache write-back
        // is needed to hand the partial to the workgroup that merges the splits
        store_through<CPL>(out + CPL * lane, num);
        if (lane == 0) {
            const float ml2[2] = {M * 0.6931471805599453f, L};
            store_through<2>(out + HD, ml2);
        }
    }
    WQ_STAMP(5);
    if (!a.fused) return;

    // ---- the last workgroup of (b, kvh) to get here merges the partials of all splits, in split order; head by head:
    //      head r's partial was written by wavefront r alone, so wavefront r reports in for it on a counter of its own
    //      and, if it is the last to do so, merges head r, without a word to the other wavefronts ----
    // The partial was stored with device-scope stores, which go through to memory.  The wavefront waits until the
    // memory system has acknowledged its stores (vmcnt(0): what a fence of narrower scope does not make the compiler
    // emit) and only then counts itself, so the wavefront that finds itself last reads partials that have arrived, with
    // device-scope loads that do not stop at a cache.  This costs one memory round trip; a device-scope release fence
    // would add a write-back of the whole L2 (measured: 19 us per call).
    bool last = false;
    if (wave < a.rep) {
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        WQ_STAMP(56);
        unsigned* const counter = a.arrive + unit * WQ_ARRIVE_STRIDE + wave;
        static_assert(WQ_ARRIVE_STRIDE >= WQ_MAX_REP, "one counter per head inside a unit's piece");
        unsigned old = 0u;
        if (lane == 0) old = __hip_atomic_fetch_add(counter, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        last = (unsigned)__builtin_amdgcn_readfirstlane((int)old) == (unsigned)S - 1u;
        WQ_STAMP(57);
        if (last && lane == 0) __hip_atomic_store(counter, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);   // for the next launch
    }
    // What follows runs once per (b, kvh, head) while the rest of the chip waits, and a wavefront's vector instruction
    // takes four cycles: every instruction counts.  Lane s holds (m, l) of split s (the launch takes this path with at
    // most 64 splits), the weights come from reductions inside the wavefront, lane s's weight is read back as a scalar
    // for the sum over the splits; no LDS, no barrier.  The partials are read through a buffer descriptor, whose range
    // check returns zero beyond the last split.
    if (last) {
        const int np = S;                          // (the splits are all the partials there are in a launch that merges them itself)
        const unsigned pbytes = (unsigned)pstride * 4u;
        const __amdgpu_buffer_rsrc_t parts = __builtin_amdgcn_make_buffer_rsrc(pbase, 0, np * (int)pbytes, 0x00020000);
        const unsigned row = (unsigned)(wave * (HD + 2)) * 4u;
        const floatx2 ml = ld_part<2>(parts, (unsigned)lane * pbytes + row + HD * 4u);
        const float m_s = lane < np ? ml[0] : -INFINITY, l_s = ml[1];
        float w_s = 0.f, M = -INFINITY, L = 0.f;
        float acc[CPL];
#pragma unroll
        for (int c = 0; c < CPL; c++) acc[c] = 0.f;
        const unsigned chan = row + (unsigned)lane * (CPL * 4u);
#pragma unroll 1
        for (int k0 = 0; k0 < np; k0 += 16) {      // 16 splits at a time: their loads are in flight together
            typename FloatN<CPL>::type pre[16];
#pragma unroll
            for (int k = 0; k < 16; k++) pre[k] = ld_part<CPL>(parts, chan + (unsigned)(k0 + k) * pbytes);
            if (k0 == 0) merge_weights_lanes(m_s, l_s, w_s, M, L);
#pragma unroll
            for (int k = 0; k < 16; k++) {
                const float wk = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, w_s), k0 + k));   // 0 beyond the last split
#pragma unroll
                for (int c = 0; c < CPL; c++) acc[c] = fmaf(part_elem<CPL>(pre[k], c), wk, acc[c]);
            }
        }
        WQ_STAMP(58);
        const int hq = kvh * a.rep + wave;
        float o[CPL];
#pragma unroll
        for (int c = 0; c < CPL; c++) o[c] = L > 0.f ? acc[c] / L : 0.f;
        store_plain<CPL>(a.out + ((int64_t)b * a.Hq + hq) * HD + CPL * lane, o);
        if (a.lse && lane == 0) a.lse[(int64_t)b * a.Hq + hq] = L > 0.f ? M + logf(L) : -INFINITY;
    }
    WQ_STAMP(59);
    finish_append(a, b, kvh, split, new_row);
}

}  // namespace
