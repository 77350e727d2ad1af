/*
 * wq.h -- C ABI of the WindowQuant hot path on AMD MI355X (gfx950).
 *
 * WindowQuant (window-adaptive mixed-precision KV-cache quantization for video-language models)
 * has three data-parallel stages; this library implements them as four calls:
 *
 *   wq_window_scores     window-level quantization search, scoring   (Sec. 3.2.1, similarity equation)
 *   wq_assign_bits       ... and bit-width decision per window        (Sec. 3.2.1 threshold rule, Sec. 3.2.2
 *                                                                      first-window pin; rank/quota rule)
 *   wq_reorder_quantize  window-level KV cache computation, prefill   (Sec. 3.3.1, Sec. 3.3.3, Alg. 2 first half)
 *   wq_decode_attention  ... and decoding over the mixed cache        (Alg. 2 second half, Sec. 3.3.2)
 *
 * Conventions
 *   - Every pointer named "dev" or documented as device memory is a HIP device pointer on the current
 *     device; every scalar and the structs themselves live on the host.  The library reads no device
 *     table on the host and never synchronises: each call only enqueues kernels on the context's stream.
 *   - The caller owns every buffer.  The library allocates nothing after wq_create (and nothing at all
 *     when wq_create is given a workspace).
 *   - Every call returns WQ_OK (0) or a negative wq_status; it never aborts.  Host-checkable argument
 *     errors are reported before anything is enqueued; wq_last_error() gives a message.
 *   - Conditions only visible on the device (a class buffer too small for what the bit assignment
 *     produced) set a bit in a device status word that wq_device_status() reads back.
 *   - Shapes: head_dim hd in {64, 128}; group in {32, 64, 128} dividing hd; Hq a multiple of Hkv with
 *     Hq/Hkv <= 8.  Anything else is WQ_ERR_UNSUPPORTED.
 *
 * Sequences and windows
 *   A batch has B sequences.  Sequence b has win_off[b+1]-win_off[b] windows of win_size[b] tokens
 *   (Sec. 3.2.1: W_i = {v_{iS} .. v_{iS+S-1}}, floor(M/S) windows).  Visual tokens that do not fill a
 *   window, text tokens and generated tokens stay 16-bit (Sec. 3.1).
 *
 * Bit classes
 *   class 0,1,2 = 2,4,8-bit codes; the 16-bit segment holds everything else.  In memory the order is
 *   2-bit, 4-bit, 8-bit, 16-bit (the order of Alg. 2, with the appendable 16-bit block last); inside a
 *   class windows keep ascending index (Alg. 2 appends in index order).
 *
 * Quantization (Sec. 3.3.3, asymmetric round-to-nearest, unsigned range [0, 2^b-1])
 *   A group is `group` consecutive channels of one token of one KV head.  With lo/hi the group's
 *   min/max, all in fp32 without fused multiply-add:
 *       m = f16(lo);  s = f16((hi - m) / (2^b-1));  if (s == 0) s = 1;  inv = 1.0f / s;
 *       code = clamp((int)rint((x - m) * inv), 0, 2^b-1)          (ties to even)
 *   and the value a code stands for is  m + s*code.  s and m are stored as IEEE binary16.
 *   Inputs must be finite with |x| <= 65504.
 *
 * Storage layout of a class buffer (b = bits, G = hd/group, cap = capacity in tokens, a multiple of 32)
 *   codes : bytes [plane][Hkv][cap*hd*b/8], plane 0 = K, 1 = V.  Codes are b-bit fields; field n of a
 *           tile/block sits at bit n*b (low bits of low bytes first).
 *           K plane, tiles of 16 tokens: token m of the tile, channel ch = j*(hd/4)+e
 *                    -> n = (j*16 + m)*(hd/4) + e
 *           V plane, blocks of 32 tokens: token u of the block, channel ch = 16*ct + mm
 *                    -> jj = (u%16)/4, tau = 4*(u/16) + u%4,  n = ((jj*16 + mm)*(hd/16) + ct)*8 + tau
 *           (both are exactly the per-lane operand order of the 16x16x32 matrix instruction, so a
 *           wavefront reads whole tiles with one coalesced load per lane and no shuffles).
 *   meta  : uint32 [plane][Hkv][cap/16][G][16]; low half = f16 s, high half = f16 m of (token, group).
 *   Sequence b owns tokens cls_off[c][b] .. cls_off[c][b]+cls_len[c][b]-1 of class c; cls_off entries are
 *   multiples of 32 and the padding up to the next multiple of 32 holds zero codes and zero metadata.
 *   16-bit segment: k16/v16 [cap16][Hkv][hd] elements of dtype16, sequence b at rows
 *   off16[b] .. off16[b]+len16[b]-1; 16-bit windows first (index order), then the video tail and text
 *   in their original order; the caller appends generated tokens and bumps len16[b] (Sec. 2.2).
 */
#ifndef WQ_H
#define WQ_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct wq_ctx wq_ctx;

typedef enum { WQ_F32 = 0, WQ_BF16 = 1, WQ_F16 = 2 } wq_dtype;
typedef enum { WQ_OK = 0, WQ_ERR_ARG = -1, WQ_ERR_UNSUPPORTED = -2, WQ_ERR_HIP = -3, WQ_ERR_WORKSPACE = -4 } wq_status;
typedef enum { WQ_SCORE_AUTO = 0, WQ_SCORE_PAIRWISE_MFMA = 1, WQ_SCORE_POOLED = 2 } wq_score_algo;
typedef enum { WQ_MODE_QUOTA = 0, WQ_MODE_THRESHOLD = 1 } wq_assign_mode;
typedef enum { WQ_DECODE_AUTO = 0, WQ_DECODE_GENERIC = 1, WQ_DECODE_MFMA = 2 } wq_decode_algo;
/* or-ed into algo: every wavefront of the matrix-core kernel gets a fixed share of the token axis, so that the
 * summation order, and with it every bit of the result, is the same on every run.  Without it the wavefronts of a
 * workgroup take the blocks of the workgroup's share one by one as they get free (faster; results agree to
 * rounding).                                                                                                   */
#define WQ_DECODE_FIXED_SHARES 0x200
/* or-ed into algo, for batches whose sequences differ a lot in length: a sequence uses ceil(num_splits * tokens /
 * max_seq_tokens) of the launch's splits (at least one; the workgroups beyond them return at once), and num_splits = 0 picks
 * wq_auto_splits_ragged instead of wq_auto_splits.  Needs max_seq_tokens > 0: the length of the longest sequence (a value
 * below it only makes more sequences use all splits).  Has an effect only where the matrix-core kernel merges its splits
 * itself (the launches that can also append); elsewhere every sequence uses all splits.                              */
#define WQ_DECODE_BY_LENGTH 0x400
/* or-ed into algo: the splits are merged by a second kernel instead of by the decode kernel's last workgroup per
 * (sequence, KV head) (what the library does by itself when a launch has more than 64 splits: the in-kernel merge holds
 * one split per lane of a wavefront).
 * Both merges do the same arithmetic in the same order: with WQ_DECODE_FIXED_SHARES their results agree bit for bit.   */
#define WQ_DECODE_SEPARATE_MERGE 0x800

/* device status bits (wq_device_status) */
#define WQ_DEV_CLASS_OVERFLOW 1u /* a class segment did not fit its cap[c]; the excess was not written    */
#define WQ_DEV_SEG16_OVERFLOW 2u /* 16-bit rows of a sequence exceeded off16[b+1]-off16[b] or cap16        */
#define WQ_DEV_TOO_MANY_WINDOWS 16u /* a sequence has more windows than the max_windows given to wq_assign_bits, wq_vote_bits or
                                  * wq_validate_assignment; the windows beyond the bound were left out                  */
#define WQ_DEV_BAD_ASSIGNMENT 32u /* wq_validate_assignment: perm is not a permutation of a sequence's windows, or its four
                                  * class counts do not add up to the number of its windows                             */
#define WQ_DEV_APPEND_TIMEOUT 4u /* wq_decode_append_attention: the workgroup that raises len16[b] gave up waiting (4 s) for
                                  * the sequence's other workgroups to start; len16[b] was raised all the same, the
                                  * workspace header may hold a stale count and must be zeroed before its next use     */

/* ---- context ----------------------------------------------------------------------------------------------
 * hip_stream   : a hipStream_t (NULL = the default stream); all work of this context is enqueued on it.
 * workspace    : device memory of workspace_bytes that the library may scribble on, or NULL to let
 *                wq_create allocate workspace_bytes itself (freed by wq_destroy).  Size it with
 *                wq_workspace_bytes; calls that need more return WQ_ERR_WORKSPACE.
 *                A caller-provided workspace must start with 16384 zero bytes (device status word and
 *                reserved words; the library leaves them zero after every call).
 * wq_create touches no GPU when it is given a workspace (or workspace_bytes == 0).                          */
int wq_create(wq_ctx** out, void* hip_stream, void* workspace, size_t workspace_bytes);
int wq_destroy(wq_ctx* ctx);
int wq_set_stream(wq_ctx* ctx, void* hip_stream);
const char* wq_last_error(const wq_ctx* ctx);
/* Blocks until the stream drains, then returns the device status word in *bits and clears it. */
int wq_device_status(wq_ctx* ctx, uint32_t* bits);

/* Host-only, pure.  Workspace needed by the largest call with these bounds (any argument may be 0). */
size_t wq_workspace_bytes(int B, int Hq, int hd, int max_splits, int64_t total_vis, int64_t total_txt, int D);
/* Host-only, pure.  Bytes of codes (return value) and metadata (*meta_bytes) of one class buffer with
 * capacity cap_tokens (rounded up to 32 here), both planes and all KV heads.  0 on unsupported shapes.      */
size_t wq_packed_bytes(int bits, int64_t cap_tokens, int Hkv, int hd, int group, size_t* meta_bytes);
/* Host-only, pure.  Split count wq_decode_attention picks for num_splits = 0 when the sequences are about equally long. */
int wq_auto_splits(int B, int Hkv, int64_t max_seq_tokens);
/* Host-only, pure.  ... and what it picks under WQ_DECODE_BY_LENGTH: total_tokens (all sequences together; the decode calls
 * take the sum of the cache's capacities for it) below 3/4 of B * max_seq_tokens gives more splits, of which a sequence
 * then uses its share by length: about twice as many workgroups have work as for equal lengths.  Never less than
 * wq_auto_splits; a workspace sized for this count lets the decode calls use it, one sized for wq_auto_splits makes them
 * fall back to that count.                                                                                          */
int wq_auto_splits_ragged(int B, int Hkv, int64_t max_seq_tokens, int64_t total_tokens);

/* ---- a1: window scores (Sec. 3.2.1) ----------------------------------------------------------------------
 * score[i] = 1/(S N) sum_{k in window i} sum_j cos(t_j, w_k), cosine := 0 for a zero vector.
 * vis_emb [total_vis, D], txt_emb [total_txt, D]  device, row-major, element type `dtype`
 * vis_off, txt_off [B+1], win_size [B], win_off [B+1]   device int32; window i of sequence b covers rows
 *          vis_off[b] + i*win_size[b] .. + win_size[b]-1
 * total_vis, total_txt, total_win : host copies of vis_off[B], txt_off[B], win_off[B] (grid bounds)
 * algo    : WQ_SCORE_POOLED uses the identity score = (mean_j t_j/|t_j|) . (mean_k w_k/|w_k|) and reads each
 *           embedding once (HBM-bound); WQ_SCORE_PAIRWISE_MFMA forms the [tokens x text] product on the
 *           matrix cores (bf16/fp16 inputs only, D a multiple of 128, 16-byte aligned embeddings, at most
 *           4 GiB of text embeddings) and normalises/reduces it in the epilogue.
 * scores  [total_win] device fp32, written.   Accumulation is fp32; no atomics, results are deterministic. */
int wq_window_scores(wq_ctx* ctx, const void* vis_emb, const void* txt_emb, int dtype, int B, int D,
                     const int32_t* vis_off, const int32_t* txt_off, const int32_t* win_size, const int32_t* win_off,
                     int64_t total_vis, int64_t total_txt, int64_t total_win, int algo, float* scores);

/* ---- a2: bit-width per window ----------------------------------------------------------------------------
 * mode WQ_MODE_THRESHOLD (Sec. 3.2.1): score > T_high -> top_bits, score < T_low -> 2, else 4 (strict).
 * mode WQ_MODE_QUOTA: windows ordered by score descending, equal scores by ascending index (NaN ranks last);
 *      the first n_top get top_bits, the next n4 get 4, the rest 2; quotas are clipped to the window count.
 * pin_first (Sec. 3.2.2): window 0 gets top_bits whatever its score; under quotas it leaves the ranking and
 *      uses one slot of the highest-precision class with a non-zero quota.
 * top_bits : 8, or 16 to keep the top tier unquantized as the paper does.
 * scores [total_win] fp32, win_off [B+1], quota [B,3] = {n_top, n4, n2} int32 (quota mode),
 * thresholds [B,2] = {T_low, T_high} fp32 (threshold mode): device.  max_windows: host bound on windows per
 * sequence (<= 8192); a sequence with more raises WQ_DEV_TOO_MANY_WINDOWS and gets only its first max_windows windows assigned.   Outputs (device): bits [total_win] uint8; perm [total_win] int32, per sequence the
 * window indices of class 2, then 4, 8, 16, each ascending; seg_windows [B,4] counts {n2,n4,n8,n16}.        */
int wq_assign_bits(wq_ctx* ctx, const float* scores, int B, const int32_t* win_off, int max_windows, int mode,
                   const int32_t* quota, const float* thresholds, int top_bits, int pin_first, uint8_t* bits,
                   int32_t* perm, int32_t* seg_windows);

/* ---- per-layer thresholds (Sec. 3.2.3 threshold functions) --------------------------------------------------
 * t_low[i] = f1(s[i]) = (e^{alpha s} - 1)/(e^alpha - 1),  t_high[i] = f2(s[i]) = (e^{-alpha s} - 1)/(e^{-alpha} - 1);
 * alpha = 0 gives the limit of both, the identity.  s[i] is layer i's hidden-state similarity in [0, 1] (the
 * caller measures it on a calibration run; the library does not).  Host-only, pure: s, t_low, t_high are host
 * arrays of n_layers entries.  Evaluated in double, returned as the fp32 values wq_assign_bits compares with.
 * WQ_ERR_ARG on NULL, n_layers < 0, a non-finite alpha or an s[i] outside [0, 1].                             */
int wq_layer_thresholds(const double* s, int n_layers, double alpha, float* t_low, float* t_high);

/* ---- batch-shared configuration (Sec. 3.2.3, last paragraph) ----------------------------------------------
 * For every window position the width that occurs most often among the sequences that have that position is
 * given to all of them; on a tie the wider one wins (the paper leaves ties open).  bits_in [total_win] uint8 as
 * written by wq_assign_bits; win_off [B+1]; max_windows: host bound on windows per sequence (<= 8192).
 * Outputs as in wq_assign_bits: bits_out [total_win] (may alias bits_in), perm [total_win], seg_windows [B,4].
 * All arrays device memory.                                                                                   */
int wq_vote_bits(wq_ctx* ctx, const uint8_t* bits_in, int B, const int32_t* win_off, int max_windows,
                 uint8_t* bits_out, int32_t* perm, int32_t* seg_windows);

/* ---- debug aid: validate an assignment on the device -----------------------------------------------------------
 * wq_reorder_quantize trusts perm and seg_windows (it gathers whatever rows perm names).  This call checks, per
 * sequence, that perm[win_off[b] .. win_off[b+1]) is a permutation of 0 .. W_b-1 and that seg_windows[b][0..3] are
 * non-negative and add up to W_b, and raises WQ_DEV_BAD_ASSIGNMENT (wq_device_status) otherwise.  One small launch; meant
 * for tables that do not come straight from wq_assign_bits / wq_vote_bits.  max_windows as in wq_assign_bits.            */
int wq_validate_assignment(wq_ctx* ctx, int B, const int32_t* win_off, int max_windows, const int32_t* perm,
                           const int32_t* seg_windows);

/* ---- packed mixed-precision cache of one layer (layout: see the header comment) -------------------------- */
typedef struct {
    int32_t B, Hkv, hd, group;
    int32_t dtype16;       /* WQ_BF16 or WQ_F16: element type of k16/v16                                   */
    int32_t reserved;
    void* codes[3];        /* device, wq_packed_bytes(bits, cap[c], ...) bytes each                         */
    void* meta[3];         /* device                                                                        */
    int64_t cap[3];        /* host: capacity in tokens per (plane, head), multiple of 32                    */
    int32_t* cls_off[3];   /* device [B+1], written by wq_reorder_quantize                                  */
    int32_t* cls_len[3];   /* device [B],   written by wq_reorder_quantize                                  */
    void* k16;             /* device [cap16][Hkv][hd]                                                       */
    void* v16;
    int64_t cap16;         /* host                                                                          */
    int32_t* off16;        /* device [B+1], set by the caller: first row of each sequence, [B] = end        */
    int32_t* len16;        /* device [B], written by wq_reorder_quantize, bumped by the caller on append    */
    float* v_scale_max;    /* device [wq_v_scale_floats(B, Hkv, cap)]: entry b, written by wq_reorder_quantize (and
                            * set to 0 by wq_dequantize in its destination, where B entries are enough), is the largest
                            * scale of a value (V) group among sequence b's quantized tokens, 0 if it has none: the
                            * matrix-core decode kernel places its fp16 weights by it.  The entries behind the first
                            * B (one per 32-token block and KV head) are wq_reorder_quantize's scratch for finding it */
} wq_packed_kv;

/* Host-only, pure: number of floats of a cache's v_scale_max table (cap: the three class capacities in tokens). */
size_t wq_v_scale_floats(int B, int Hkv, const int64_t cap[3]);

/* ---- a3: reorder + quantize + pack (Alg. 2, prefill half) ------------------------------------------------
 * K, V [total_rows, Hkv, hd] device, element type `dtype`; sequence b owns rows kv_off[b]..kv_off[b+1]-1:
 * its windows first, then tail and text rows (kept 16-bit).  bits/perm/seg_windows as written by
 * wq_assign_bits.  dtype16 must be WQ_BF16 for bf16 input, WQ_F16 for fp16 and fp32 input (fp32 values are
 * rounded to nearest even).  total_rows: host copy of kv_off[B]; with total_rows > 0, K, V and perm must not be NULL
 * (perm is not read when the batch has no window at all: any valid pointer will do).  Fills every field of *out marked
 * "written"; all of out's pointers and capacities are set by the caller.                                    */
int wq_reorder_quantize(wq_ctx* ctx, const void* K, const void* V, int dtype, int B, const int32_t* kv_off,
                        const int32_t* win_size, const int32_t* win_off, const int32_t* perm,
                        const int32_t* seg_windows, int64_t total_rows, const wq_packed_kv* out);

/* ---- appending a generated token (Sec. 2.2: new keys and values go to the end of the cache; Sec. 3.1: generated
 * tokens stay 16-bit) --------------------------------------------------------------------------------------
 * Writes k_new, v_new [B, Hkv, hd] (device, element type `dtype`) as row off16[b]+len16[b] of sequence b's
 * 16-bit segment and adds one to len16[b] (on the device, in stream order).  dtype pairs with dtype16 as in
 * wq_reorder_quantize (fp32 values are rounded to fp16, nearest even).  A sequence whose segment is full
 * (off16[b]+len16[b] == off16[b+1], or == cap16) is left unchanged and WQ_DEV_SEG16_OVERFLOW is raised.       */
int wq_append_kv(wq_ctx* ctx, const void* k_new, const void* v_new, int dtype, int B, const wq_packed_kv* kv);

/* ---- a decode step in one call (Sec. 2.2): append the generated token's keys and values, then attend over the
 * cache that now includes them.  Same arguments and results as wq_append_kv(k_new, v_new, new_dtype) followed by
 * wq_decode_attention(...).  When the matrix-core kernel handles the whole launch (what WQ_DECODE_AUTO picks for
 * hd/group == 2 with a query of the cache's 16-bit type family), k_new, v_new have the cache's own 16-bit type and there
 * are at most 64 splits, it is ONE kernel launch: the new row is read from k_new / v_new by the workgroup that walks its block, copied into the cache
 * by another, and len16[b] is raised by the sequence's last workgroup to finish; otherwise the two launches are made.
 * A sequence whose 16-bit segment is full is attended without the new token and raises WQ_DEV_SEG16_OVERFLOW.
 * WQ_DECODE_PARTIALS_ONLY is not accepted here.                                                                  */
int wq_decode_append_attention(wq_ctx* ctx, const void* q, int q_dtype, int B, int Hq, const wq_packed_kv* kv,
                               const void* k_new, const void* v_new, int new_dtype, float sm_scale, int num_splits,
                               int64_t max_seq_tokens, int algo, float* out, float* lse);

/* ---- the unfused variant of the operator-fusion ablation (operator fusion: Sec. 3.3.3; its ablation: Sec. 4.4, table on the impact of operator fusion) ------------------
 * Dequantizes a packed cache to memory: sequence b's rows off16[b] .. of dst's 16-bit segment receive the values
 * m + s*code (one fp32 fused multiply-add, rounded to nearest even into dtype16) of src's 2-bit, 4-bit and 8-bit
 * tokens, in this order (the order of the cache), followed by src's 16-bit rows; dst's len16 is written, dst's
 * classes are made empty (cls_len = 0, cls_off = 0).  wq_decode_attention over dst is then plain 16-bit attention
 * over the dequantized cache: what an implementation without the fused kernel runs at every decode step.
 * src, dst: same B, Hkv, hd, dtype16; dst's tables and 16-bit segment are the caller's (its class capacities may be
 * 0).  A sequence that does not fit dst's rows (off16[b+1]-off16[b], cap16) gets len16 = 0 and raises
 * WQ_DEV_SEG16_OVERFLOW.                                                                                         */
int wq_dequantize(wq_ctx* ctx, int B, const wq_packed_kv* src, const wq_packed_kv* dst);

/* ---- a4: decode attention over the packed cache (Alg. 2, decode half) -------------------------------------
 * out[b,h,:] = sum_t softmax_t(sm_scale * q[b,h].k^_t) v^_t over the 2-, 4-, 8- and 16-bit segments of
 * sequence b, one softmax over all of them, no mask (Sec. 2.1); head h reads KV head h/(Hq/Hkv).
 * Codes are expanded in registers; the token axis is split over num_splits workgroups per (b, KV head)
 * and merged by log-sum-exp in a fixed order (no float atomics).  Which wavefront sums which tokens is fixed
 * only under WQ_DECODE_FIXED_SHARES.
 * q [B,Hq,hd] device, element type q_dtype; out [B,Hq,hd] device fp32; lse [B,Hq] device fp32 or NULL
 * (natural-log sum of exp of the scaled logits).  num_splits 0 = automatic (wq_auto_splits).  max_seq_tokens: host
 * bound on tokens of any one sequence (used by the automatic split and by WQ_DECODE_BY_LENGTH; a wrong value costs speed,
 * not correctness).  algo: WQ_DECODE_AUTO picks the
 * matrix-core kernel when hd/group == 2, else the generic one.  Limits (WQ_ERR_UNSUPPORTED beyond them): Hq a
 * multiple of Hkv with at most 8 query heads per KV head, hd 64 or 128, group 32, 64 or 128, B at most 65535, and for
 * the matrix-core kernel at most 2^27 token slots in the cache (cap[0] + cap[1] + cap[2] + cap16: it cuts the workgroups'
 * shares on a 32-bit cost axis); num_splits above 1024 is WQ_ERR_ARG.
 * Value range: the matrix-core kernel multiplies the softmax weights (at most 32 relative to its running reference) with
 * the scales of the value groups in fp16.  It places that product by the sequence's largest value scale (v_scale_max[b] of
 * the cache, which wq_reorder_quantize writes): the largest product is 2^14..2^15 whatever the values' magnitude, so nothing
 * overflows for any scale that fp16 holds, and a token's weight is lost to fp16's subnormal range only when it is below
 * 2^-29 of the largest one (times the ratio of the sequence's largest value scale to the token's own: a group of small
 * values next to groups of large ones loses more, of a contribution that is small by the same ratio).  A cache filled by
 * other means than wq_reorder_quantize must set v_scale_max[b] itself (an upper bound will do; too large a bound costs
 * range at the bottom).  Keys have no such limit.  */
int wq_decode_attention(wq_ctx* ctx, const void* q, int q_dtype, int B, int Hq, const wq_packed_kv* kv,
                        float sm_scale, int num_splits, int64_t max_seq_tokens, int algo, float* out, float* lse);

/* ---- decode attention for callers that cannot allocate -------------------------------------------------------
 * For code that must not call hipMalloc: kernels enqueued under HIP graph capture, tight serving loops, harnesses
 * that forbid allocation.  Same arguments, results and limits as wq_decode_attention, without a context and without
 * a workspace: the split-K partials, the decode kernel's counters and the device status word live in a device array
 * of WQ_STATIC_SCRATCH_BYTES that is part of the library's code object (one copy per GPU, held until the process
 * ends).  hip_stream: a hipStream_t (NULL = the default stream) of the current device.  The call allocates nothing
 * (no hipMalloc, no hipFree, no allocating library routine) and does not synchronise.
 * A call that needs more than the array holds (wq_workspace_bytes(B, Hq, hd, num_splits, 0, 0, 0) bytes: more sequences,
 * heads or splits) returns WQ_ERR_WORKSPACE and enqueues nothing; wq_static_last_error() says how much it asked for.
 * Every call on a GPU shares that GPU's array and the array keeps what the last call left in it: the decode kernel leaves
 * its counters zero when it ends and reads no partial that it has not written, so calls in stream order need no clearing in between;
 * calls that overlap on one GPU (two streams, two threads) race on it and must not be made.                          */
#define WQ_STATIC_SCRATCH_BYTES (8u << 20)
int wq_decode_attention_static(void* hip_stream, const void* q, int q_dtype, int B, int Hq, const wq_packed_kv* kv,
                               float sm_scale, int num_splits, int64_t max_seq_tokens, int algo, float* out, float* lse);
/* message of the last wq_decode_attention_static error on the current device (host string, valid until the next call) */
const char* wq_static_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* WQ_H */
