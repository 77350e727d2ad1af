/*
 * WindowQuant CPU oracle  --  TEST INFRASTRUCTURE, NOT PRODUCT CODE.
 *
 * A plain, slow, obviously-correct implementation of what the WindowQuant hot
 * path computes, written from the paper's definitions.  Only tests, the smoke
 * check and the benchmark's cpu_baseline leg may build, load or call it; the
 * GPU library never does and shares no source, header, table or helper with it.
 *
 *   O1  window/text similarity          Sec. 3.2.1, similarity equation
 *   O2  bit-width assignment            Sec. 3.2.1 (threshold rule), Sec. 3.2.2
 *                                       (first-window pin), Alg. 2 prefill loop
 *                                       (stable class order); rank/quota rule of
 *                                       the build's problem statement
 *   O3  reorder + asymmetric RTN        Sec. 3.3.1, Sec. 3.3.3, Alg. 2 prefill half
 *   O4  mixed-precision decode attention  Alg. 2 decode half, Sec. 3.3.2
 *   (wq_oracle.py adds two small host-side steps in plain Python: the per-layer threshold functions f1, f2 of
 *   Sec. 3.2.3 and the batch-shared configuration by majority vote of the same section's last paragraph.)
 *
 * Floating point is fp64 everywhere except O3, whose integer codes are defined
 * by an explicit fp32 operation sequence (the paper fixes "round to nearest";
 * the build fixes fp32, ties-to-even, no fused multiply-add).  Build with
 *     gcc -O2 -ffp-contract=off -fno-fast-math
 * Pins (tests, CPU only): f16 conversion vs numpy.float16; O1 pairwise form vs
 * pooled identity vs hand-computed tiny case; O2 sort form vs counting form;
 * O3 error bound, end points, constant groups, the paper's byte count for its
 * 100-frame token mix; O4 reorder invariance, textbook softmax(qK^T)V for an
 * all-16-bit cache, uniform keys, one-hot logits, GQA duplication.
 * Parity unpinned: none of the four functions lacks a pin; absolute values are
 * pinned only through those definitions (the paper prints no worked example).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

/* ------------------------------------------------------------------------ */
/* IEEE binary16 <-> binary32, round-to-nearest-even, by bit manipulation     */
/* ------------------------------------------------------------------------ */
uint16_t wqo_f32_to_f16_bits(float f)
{
    uint32_t u;
    memcpy(&u, &f, 4);
    uint32_t sign = (u >> 16) & 0x8000u;
    uint32_t ex = (u >> 23) & 0xFFu;
    uint32_t man = u & 0x7FFFFFu;
    if (ex == 0xFFu)                              /* inf / nan */
        return (uint16_t)(sign | 0x7C00u | (man ? 0x200u : 0u));
    int e = (int)ex - 127 + 15;                   /* biased half exponent */
    if (e >= 31)
        return (uint16_t)(sign | 0x7C00u);        /* overflow -> inf */
    if (e <= 0) {                                 /* result is subnormal or zero */
        int shift = 14 - e;                       /* to units of 2^-24 */
        if (shift > 24)
            return (uint16_t)sign;
        uint32_t m24 = man | 0x800000u;
        uint32_t h = m24 >> shift;
        uint32_t rem = m24 & ((1u << shift) - 1u);
        uint32_t half = 1u << (shift - 1);
        if (rem > half || (rem == half && (h & 1u)))
            h++;
        return (uint16_t)(sign | h);
    }
    uint32_t h = ((uint32_t)e << 10) | (man >> 13);
    uint32_t rem = man & 0x1FFFu;
    if (rem > 0x1000u || (rem == 0x1000u && (h & 1u)))
        h++;                                      /* a carry may reach inf: correct */
    return (uint16_t)(sign | h);
}

double wqo_f16_bits_to_f64(uint16_t h)
{
    int sign = (h >> 15) & 1;
    int e = (h >> 10) & 0x1F;
    int man = h & 0x3FF;
    double v;
    if (e == 0)
        v = ldexp((double)man, -24);
    else if (e == 31)
        v = man ? NAN : INFINITY;
    else
        v = ldexp((double)(man | 0x400), e - 25);
    return sign ? -v : v;
}

/* ------------------------------------------------------------------------ */
/* O1  similarity of each window with the text prompt (Sec. 3.2.1)            */
/*     sim(T, W_i) = 1/(S N) * sum_j sum_k  t_j.w_k / (|t_j| |w_k|)            */
/*     A zero-norm token contributes 0 to every pair it is in.                */
/* ------------------------------------------------------------------------ */
static double dotd(const float *a, const float *b, int D)
{
    double s = 0.0;
    for (int d = 0; d < D; d++)
        s += (double)a[d] * (double)b[d];
    return s;
}

/* literal form: every (text token, window token) pair */
void wqo_scores_pairwise(const float *Ev, const float *Et, int D, int B, const int32_t *vis_off,
                         const int32_t *txt_off, const int32_t *win_size, const int32_t *win_off,
                         double *scores)
{
    for (int b = 0; b < B; b++) {
        int S = win_size[b], W = win_off[b + 1] - win_off[b];
        int N = txt_off[b + 1] - txt_off[b];
        const float *T = Et + (int64_t)txt_off[b] * D;
#pragma omp parallel for schedule(dynamic)
        for (int i = 0; i < W; i++) {
            double acc = 0.0;
            for (int k = 0; k < S; k++) {
                const float *w = Ev + ((int64_t)vis_off[b] + (int64_t)i * S + k) * D;
                double nw = sqrt(dotd(w, w, D));
                for (int j = 0; j < N; j++) {
                    const float *t = T + (int64_t)j * D;
                    double nt = sqrt(dotd(t, t, D));
                    if (nw > 0.0 && nt > 0.0)
                        acc += dotd(t, w, D) / (nt * nw);
                }
            }
            scores[win_off[b] + i] = (S > 0 && N > 0) ? acc / ((double)S * (double)N) : 0.0;
        }
    }
}

/* same quantity by linearity: (mean_j t_j/|t_j|) . (mean_k w_k/|w_k|) */
void wqo_scores_pooled(const float *Ev, const float *Et, int D, int B, const int32_t *vis_off,
                       const int32_t *txt_off, const int32_t *win_size, const int32_t *win_off,
                       double *scores)
{
    double *tbar = (double *)malloc(sizeof(double) * (size_t)D);
    for (int b = 0; b < B; b++) {
        int S = win_size[b], W = win_off[b + 1] - win_off[b];
        int N = txt_off[b + 1] - txt_off[b];
        for (int d = 0; d < D; d++)
            tbar[d] = 0.0;
        for (int j = 0; j < N; j++) {
            const float *t = Et + ((int64_t)txt_off[b] + j) * D;
            double nt = sqrt(dotd(t, t, D));
            if (nt > 0.0)
                for (int d = 0; d < D; d++)
                    tbar[d] += (double)t[d] / nt;
        }
        for (int d = 0; d < D && N > 0; d++)
            tbar[d] /= (double)N;
#pragma omp parallel for schedule(dynamic)
        for (int i = 0; i < W; i++) {
            double acc = 0.0;
            for (int k = 0; k < S; k++) {
                const float *w = Ev + ((int64_t)vis_off[b] + (int64_t)i * S + k) * D;
                double nw = sqrt(dotd(w, w, D));
                if (nw > 0.0) {
                    double p = 0.0;
                    for (int d = 0; d < D; d++)
                        p += tbar[d] * (double)w[d];
                    acc += p / nw;
                }
            }
            scores[win_off[b] + i] = (S > 0 && N > 0) ? acc / (double)S : 0.0;
        }
    }
    free(tbar);
}

/* ------------------------------------------------------------------------ */
/* O2  bit-width per window, stable class order                               */
/*   mode 1 (paper, Sec. 3.2.1): score > T_high -> top, score < T_low -> 2,    */
/*           else 4 (strict inequalities, equality -> 4).                     */
/*   mode 0 (rank/quota): order windows by score descending, ties by lower    */
/*           index first; first n_top -> top, next n4 -> 4, rest -> 2.        */
/*           Quotas are clipped to the number of windows in that order.        */
/*           NaN ranks as -infinity.                                           */
/*   pin (Sec. 3.2.2): window 0 always gets the top width.  Under quotas it    */
/*           leaves the ranking and uses one slot of the highest-precision     */
/*           class whose quota is non-zero, so the mix stays as requested.     */
/*   perm  : windows of class 2 in ascending index, then 4, then 8, then 16    */
/*           (Alg. 2's prefill loop appends in index order).                   */
/* ------------------------------------------------------------------------ */
typedef struct {
    float key;
    int idx;
} rank_item;

static int rank_cmp(const void *a, const void *b)
{
    const rank_item *x = (const rank_item *)a, *y = (const rank_item *)b;
    if (x->key > y->key)
        return -1;
    if (x->key < y->key)
        return 1;
    return (x->idx > y->idx) - (x->idx < y->idx);
}

void wqo_assign_bits(const float *scores, int B, const int32_t *win_off, int mode, const int32_t *quota,
                     const float *thresholds, int top_bits, int pin_first, uint8_t *bits, int32_t *perm,
                     int32_t *seg_windows)
{
    static const int class_bits[4] = {2, 4, 8, 16};
    for (int b = 0; b < B; b++) {
        int W = win_off[b + 1] - win_off[b];
        const float *s = scores + win_off[b];
        uint8_t *bt = bits + win_off[b];
        if (mode == 1) {
            float lo = thresholds[2 * b], hi = thresholds[2 * b + 1];
            for (int i = 0; i < W; i++)
                bt[i] = (uint8_t)(s[i] > hi ? top_bits : (s[i] < lo ? 2 : 4));
            if (pin_first && W > 0)
                bt[0] = (uint8_t)top_bits;
        } else {
            int n_top = quota[3 * b], n4 = quota[3 * b + 1];
            rank_item *it = (rank_item *)malloc(sizeof(rank_item) * (size_t)(W > 0 ? W : 1));
            int n = 0;
            int first = 0;
            if (pin_first && W > 0) {
                bt[0] = (uint8_t)top_bits;
                first = 1;
                if (n_top > 0)
                    n_top--;
                else if (n4 > 0)
                    n4--;
            }
            for (int i = first; i < W; i++) {
                it[n].key = isnan(s[i]) ? -INFINITY : s[i];
                it[n].idx = i;
                n++;
            }
            qsort(it, (size_t)n, sizeof(rank_item), rank_cmp);
            if (n_top > n)
                n_top = n;
            if (n_top < 0)
                n_top = 0;
            if (n4 > n - n_top)
                n4 = n - n_top;
            if (n4 < 0)
                n4 = 0;
            for (int r = 0; r < n; r++)
                bt[it[r].idx] = (uint8_t)(r < n_top ? top_bits : (r < n_top + n4 ? 4 : 2));
            free(it);
        }
        int pos = 0;
        for (int c = 0; c < 4; c++) {
            int cnt = 0;
            for (int i = 0; i < W; i++)
                if (bt[i] == class_bits[c]) {
                    perm[win_off[b] + pos++] = i;
                    cnt++;
                }
            seg_windows[4 * b + c] = cnt;
        }
    }
}

/* second formulation of the rank rule: rank_i = #{j : s_j > s_i or (s_j == s_i and j < i)} */
void wqo_rank_by_counting(const float *s, int W, int first, int32_t *rank)
{
    for (int i = first; i < W; i++) {
        float si = isnan(s[i]) ? -INFINITY : s[i];
        int r = 0;
        for (int j = first; j < W; j++) {
            float sj = isnan(s[j]) ? -INFINITY : s[j];
            if (sj > si || (sj == si && j < i))
                r++;
        }
        rank[i] = r;
    }
}

/* ------------------------------------------------------------------------ */
/* O3  asymmetric round-to-nearest quantization of one group (Sec. 3.3.3)     */
/*   Unsigned range [0, 2^b - 1]; scale = (max - min) / (2^b - 1).  The        */
/*   zero-point is kept in its floating form, the group minimum:              */
/*        code = rne((x - m) / s),   x^ = m + s * code.                        */
/*   Exact fp32 sequence (no fused multiply-add), s and m stored as binary16:  */
/*        lo = min x (-0 counts as +0), hi = max x                             */
/*        m  = f16(lo)                  r  = hi - m                            */
/*        s  = f16(r / qmax)            if s == 0: s = 1                       */
/*        inv = 1.0f / s                                                       */
/*        code = clamp((int)rint((x - m) * inv), 0, qmax)                      */
/*   Precondition: finite inputs with |x| <= 65504.                            */
/* ------------------------------------------------------------------------ */
void wqo_quantize_group(const float *x, int n, int bits, uint8_t *codes, uint16_t *s_bits, uint16_t *m_bits)
{
    volatile float lo = x[0], hi = x[0];
    for (int i = 1; i < n; i++) {
        if (x[i] < lo)
            lo = x[i];
        if (x[i] > hi)
            hi = x[i];
    }
    if (lo == 0.0f)
        lo = 0.0f;                                /* a zero minimum is stored as +0: -0 == +0, so which of the two a search
                                                     for the minimum ends with depends on the order of its comparisons,
                                                     and the stored bits must not */
    int qmax = (1 << bits) - 1;
    uint16_t mb = wqo_f32_to_f16_bits(lo);
    volatile float m = (float)wqo_f16_bits_to_f64(mb);
    volatile float r = hi - m;
    volatile float s0 = r / (float)qmax;
    uint16_t sb = wqo_f32_to_f16_bits(s0);
    volatile float s = (float)wqo_f16_bits_to_f64(sb);
    if (s == 0.0f) {
        s = 1.0f;
        sb = 0x3C00u;
    }
    volatile float inv = 1.0f / s;
    for (int i = 0; i < n; i++) {
        volatile float d = x[i] - m;
        volatile float t = d * inv;
        float q = rintf(t);                       /* default rounding mode: ties to even */
        int c = (int)q;
        if (q < 0.0f)
            c = 0;
        if (q > (float)qmax)
            c = qmax;
        codes[i] = (uint8_t)c;
    }
    *s_bits = sb;
    *m_bits = mb;
}

/* Padded length of a class segment: whole 32-token blocks. */
static int pad32(int n) { return (n + 31) / 32 * 32; }

/*
 * Reorder + quantize one batch (Alg. 2, prefill half).
 *   K, V      [rows, Hkv, hd] fp32 holding the cache's storage-type values; sequence b owns rows
 *             kv_off[b] .. kv_off[b+1]-1: its W_b*S_b windowed visual tokens first, then the video
 *             tail and the text tokens, which stay 16-bit (Sec. 3.1).
 *   perm/seg_windows as produced by O2.
 * Outputs, class c = 0,1,2 for 2,4,8 bits:
 *   cls_off[c][B+1], cls_len[c][B]   token offset (padded to 32) and true length of each sequence
 *   codes[c]  [2][Hkv][cap_c][hd]    logical codes, plane 0 = K, 1 = V; padding tokens are 0
 *   sbits/mbits[c] [2][Hkv][cap_c][hd/g]
 *   rows16    [cap16]                source row of every 16-bit token, sequence b at off16[b];
 *   len16[B]                         16-bit windows in index order, then tail, then text
 * The gather itself (which source row lands where) is returned as src_row[c][cap_c] (-1 = padding).
 */
void wqo_plan(int B, const int32_t *kv_off, const int32_t *win_size, const int32_t *win_off,
              const int32_t *seg_windows, int32_t *cls_off /*[3][B+1]*/, int32_t *cls_len /*[3][B]*/,
              int32_t *len16 /*[B]*/)
{
    for (int c = 0; c < 3; c++) {
        cls_off[c * (B + 1)] = 0;
        for (int b = 0; b < B; b++) {
            int n = seg_windows[4 * b + c] * win_size[b];
            cls_len[c * B + b] = n;
            cls_off[c * (B + 1) + b + 1] = cls_off[c * (B + 1) + b] + pad32(n);
        }
    }
    for (int b = 0; b < B; b++) {
        int W = win_off[b + 1] - win_off[b];
        int rows = kv_off[b + 1] - kv_off[b];
        len16[b] = seg_windows[4 * b + 3] * win_size[b] + (rows - W * win_size[b]);
    }
}

void wqo_gather_rows(int B, const int32_t *kv_off, const int32_t *win_size, const int32_t *win_off,
                     const int32_t *perm, const int32_t *seg_windows, const int32_t *cls_off,
                     const int32_t *off16, int64_t *src_row2, int64_t *src_row4, int64_t *src_row8,
                     int64_t *rows16)
{
    int64_t *dst[3] = {src_row2, src_row4, src_row8};
    for (int b = 0; b < B; b++) {
        int S = win_size[b], W = win_off[b + 1] - win_off[b];
        int pos = 0;                              /* position in perm */
        for (int c = 0; c < 3; c++) {
            int64_t o = cls_off[c * (B + 1) + b];
            for (int r = 0; r < seg_windows[4 * b + c]; r++) {
                int win = perm[win_off[b] + pos++];
                for (int k = 0; k < S; k++)
                    dst[c][o++] = (int64_t)kv_off[b] + (int64_t)win * S + k;
            }
        }
        int64_t o = off16[b];
        for (int r = 0; r < seg_windows[4 * b + 3]; r++) {
            int win = perm[win_off[b] + pos++];
            for (int k = 0; k < S; k++)
                rows16[o++] = (int64_t)kv_off[b] + (int64_t)win * S + k;
        }
        for (int64_t t = (int64_t)kv_off[b] + (int64_t)W * S; t < kv_off[b + 1]; t++)
            rows16[o++] = t;
    }
}

/* quantize the gathered rows of one class: X [rows, Hkv, hd] -> codes [Hkv][cap][hd], meta [Hkv][cap][G] */
void wqo_quantize_class(const float *X, int Hkv, int hd, int g, int bits, int64_t cap, const int64_t *src_row,
                        uint8_t *codes, uint16_t *sbits, uint16_t *mbits)
{
    int G = hd / g;
#pragma omp parallel for schedule(static)
    for (int64_t t = 0; t < cap; t++) {
        for (int h = 0; h < Hkv; h++) {
            uint8_t *c = codes + ((int64_t)h * cap + t) * hd;
            uint16_t *sb = sbits + ((int64_t)h * cap + t) * G;
            uint16_t *mb = mbits + ((int64_t)h * cap + t) * G;
            if (src_row[t] < 0) {
                memset(c, 0, (size_t)hd);
                memset(sb, 0, sizeof(uint16_t) * (size_t)G);
                memset(mb, 0, sizeof(uint16_t) * (size_t)G);
                continue;
            }
            const float *x = X + (src_row[t] * Hkv + h) * hd;
            for (int gi = 0; gi < G; gi++)
                wqo_quantize_group(x + gi * g, g, bits, c + gi * g, sb + gi, mb + gi);
        }
    }
}

/* ------------------------------------------------------------------------ */
/* Packed byte images (the build's storage format; the paper leaves the       */
/* physical packing open).  Codes are b-bit fields, little-endian: code n of  */
/* a tile sits at bit n*b of the tile (low bits of low bytes first).          */
/*  K plane: tiles of 16 tokens.  Token m (0..15), channel ch = j*(hd/4)+e    */
/*           -> n = (j*16 + m)*(hd/4) + e                                      */
/*  V plane: blocks of 32 tokens.  Token u (0..31), channel ch = 16*ct + mm   */
/*           -> jj = (u%16)/4, tau = 4*(u/16) + u%4,                           */
/*              n = ((jj*16 + mm)*(hd/16) + ct)*8 + tau                        */
/*  meta   : per tile of 16 tokens, [group][token] 32-bit words,              */
/*           low half = f16 scale, high half = f16 minimum.                   */
/* ------------------------------------------------------------------------ */
static void put_code(uint8_t *base, int64_t n, int bits, unsigned code)
{
    int64_t bit = n * bits;
    base[bit >> 3] |= (uint8_t)(code << (bit & 7));   /* fields never straddle a byte: b | 8 */
}

void wqo_pack_k(const uint8_t *codes /*[cap][hd]*/, int64_t cap, int hd, int bits, uint8_t *out)
{
    int64_t tile_bytes = (int64_t)16 * hd * bits / 8;
    memset(out, 0, (size_t)(cap / 16 * tile_bytes));
    int q = hd / 4;
    for (int64_t t = 0; t < cap; t++)
        for (int ch = 0; ch < hd; ch++) {
            int m = (int)(t % 16), j = ch / q, e = ch % q;
            put_code(out + t / 16 * tile_bytes, (int64_t)(j * 16 + m) * q + e, bits, codes[t * hd + ch]);
        }
}

void wqo_pack_v(const uint8_t *codes /*[cap][hd]*/, int64_t cap, int hd, int bits, uint8_t *out)
{
    int64_t blk_bytes = (int64_t)32 * hd * bits / 8;
    memset(out, 0, (size_t)(cap / 32 * blk_bytes));
    for (int64_t t = 0; t < cap; t++)
        for (int ch = 0; ch < hd; ch++) {
            int u = (int)(t % 32), ct = ch / 16, mm = ch % 16;
            int jj = (u % 16) / 4, tau = 4 * (u / 16) + u % 4;
            put_code(out + t / 32 * blk_bytes, ((int64_t)(jj * 16 + mm) * (hd / 16) + ct) * 8 + tau, bits,
                     codes[t * hd + ch]);
        }
}

void wqo_pack_meta(const uint16_t *sbits, const uint16_t *mbits /*[cap][G]*/, int64_t cap, int G, uint32_t *out)
{
    for (int64_t t = 0; t < cap; t++)
        for (int gi = 0; gi < G; gi++)
            out[(t / 16 * G + gi) * 16 + t % 16] = (uint32_t)sbits[t * G + gi] | ((uint32_t)mbits[t * G + gi] << 16);
}

/* ------------------------------------------------------------------------ */
/* O4  decode attention over the mixed-precision cache (Alg. 2, decode half)  */
/*   logits over the 2-, 4-, 8-bit blocks (dequantized x^ = m + s*code) and    */
/*   the 16-bit block, ONE softmax over their concatenation, weighted sum of   */
/*   the values of every block.  No mask in decoding (Sec. 2.1).  Query head   */
/*   h reads KV head h / (Hq/Hkv).  All arithmetic fp64.                       */
/* ------------------------------------------------------------------------ */
typedef struct {
    const uint8_t *codes;     /* [2][Hkv][cap][hd] */
    const uint16_t *sbits;    /* [2][Hkv][cap][G]  */
    const uint16_t *mbits;
    const int32_t *off;       /* [B+1] */
    const int32_t *len;       /* [B]   */
    int64_t cap;
} wqo_class;

void wqo_decode_attention(const float *q /*[B][Hq][hd]*/, int B, int Hq, int Hkv, int hd, int g,
                          const uint8_t *codes2, const uint16_t *s2, const uint16_t *m2, const int32_t *off2,
                          const int32_t *len2, int64_t cap2, const uint8_t *codes4, const uint16_t *s4,
                          const uint16_t *m4, const int32_t *off4, const int32_t *len4, int64_t cap4,
                          const uint8_t *codes8, const uint16_t *s8, const uint16_t *m8, const int32_t *off8,
                          const int32_t *len8, int64_t cap8, const float *k16, const float *v16 /*[cap16][Hkv][hd]*/,
                          const int32_t *off16, const int32_t *len16, double sm_scale, double *out /*[B][Hq][hd]*/,
                          double *lse /*[B][Hq] or NULL*/)
{
    wqo_class cls[3] = {{codes2, s2, m2, off2, len2, cap2}, {codes4, s4, m4, off4, len4, cap4},
                        {codes8, s8, m8, off8, len8, cap8}};
    int rep = Hq / Hkv, G = hd / g;
#pragma omp parallel for collapse(2) schedule(dynamic)
    for (int b = 0; b < B; b++)
        for (int h = 0; h < Hq; h++) {
            int kvh = h / rep;
            const float *qv = q + ((int64_t)b * Hq + h) * hd;
            int64_t T = len16[b];
            for (int c = 0; c < 3; c++)
                T += cls[c].len[b];
            double *logit = (double *)malloc(sizeof(double) * (size_t)(T > 0 ? T : 1));
            double *vhat = (double *)malloc(sizeof(double) * (size_t)(T > 0 ? T : 1) * (size_t)hd);
            int64_t n = 0;
            for (int c = 0; c < 3; c++)
                for (int t = 0; t < cls[c].len[b]; t++) {
                    int64_t row = (int64_t)kvh * cls[c].cap + cls[c].off[b] + t;
                    int64_t vrow = ((int64_t)Hkv + kvh) * cls[c].cap + cls[c].off[b] + t;
                    double acc = 0.0;
                    for (int gi = 0; gi < G; gi++) {
                        double s = wqo_f16_bits_to_f64(cls[c].sbits[row * G + gi]);
                        double m = wqo_f16_bits_to_f64(cls[c].mbits[row * G + gi]);
                        double sv = wqo_f16_bits_to_f64(cls[c].sbits[vrow * G + gi]);
                        double mv = wqo_f16_bits_to_f64(cls[c].mbits[vrow * G + gi]);
                        for (int ch = gi * g; ch < (gi + 1) * g; ch++) {
                            double khat = m + s * (double)cls[c].codes[row * hd + ch];
                            acc += (double)qv[ch] * khat;
                            vhat[n * hd + ch] = mv + sv * (double)cls[c].codes[vrow * hd + ch];
                        }
                    }
                    logit[n++] = acc * sm_scale;
                }
            for (int t = 0; t < len16[b]; t++) {
                int64_t row = ((int64_t)off16[b] + t) * Hkv + kvh;
                double acc = 0.0;
                for (int ch = 0; ch < hd; ch++) {
                    acc += (double)qv[ch] * (double)k16[row * hd + ch];
                    vhat[n * hd + ch] = (double)v16[row * hd + ch];
                }
                logit[n++] = acc * sm_scale;
            }
            double mx = -INFINITY, den = 0.0;
            for (int64_t t = 0; t < T; t++)
                if (logit[t] > mx)
                    mx = logit[t];
            double *o = out + ((int64_t)b * Hq + h) * hd;
            for (int ch = 0; ch < hd; ch++)
                o[ch] = 0.0;
            for (int64_t t = 0; t < T; t++) {
                double p = exp(logit[t] - mx);
                den += p;
                for (int ch = 0; ch < hd; ch++)
                    o[ch] += p * vhat[t * hd + ch];
            }
            for (int ch = 0; ch < hd && T > 0; ch++)
                o[ch] /= den;
            if (lse)
                lse[(int64_t)b * Hq + h] = T > 0 ? mx + log(den) : -INFINITY;
            free(logit);
            free(vhat);
        }
}

/* Textbook attention on an explicit fp32-valued cache (no quantization): used for the invariance pins. */
void wqo_attention_dense(const float *q /*[Hq][hd]*/, const float *K, const float *V /*[T][Hkv][hd]*/, int T, int Hq,
                         int Hkv, int hd, double sm_scale, double *out /*[Hq][hd]*/)
{
    int rep = Hq / Hkv;
    for (int h = 0; h < Hq; h++) {
        int kvh = h / rep;
        double *logit = (double *)malloc(sizeof(double) * (size_t)(T > 0 ? T : 1));
        double mx = -INFINITY, den = 0.0;
        for (int t = 0; t < T; t++) {
            logit[t] = sm_scale * dotd(q + (int64_t)h * hd, K + ((int64_t)t * Hkv + kvh) * hd, hd);
            if (logit[t] > mx)
                mx = logit[t];
        }
        double *o = out + (int64_t)h * hd;
        for (int ch = 0; ch < hd; ch++)
            o[ch] = 0.0;
        for (int t = 0; t < T; t++) {
            double p = exp(logit[t] - mx);
            den += p;
            for (int ch = 0; ch < hd; ch++)
                o[ch] += p * (double)V[((int64_t)t * Hkv + kvh) * hd + ch];
        }
        for (int ch = 0; ch < hd && T > 0; ch++)
            o[ch] /= den;
        free(logit);
    }
}

int wqo_num_threads(void)
{
#ifdef _OPENMP
    extern int omp_get_max_threads(void);
    return omp_get_max_threads();
#else
    return 1;
#endif
}
