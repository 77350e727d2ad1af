// C-ABI entry points of libwq: context handling, host-side argument validation, dispatch.
// Every check that needs only host data happens here, before anything is enqueued.
#include <math.h>
#include <mutex>
#include <new>
#include <string.h>

#include "wq_internal.h"

namespace {

bool shape_ok(int Hkv, int hd, int group)
{
    return Hkv > 0 && (hd == 64 || hd == 128) && (group == 32 || group == 64 || group == 128) && hd % group == 0;
}

bool dtype_ok(int d) { return d == WQ_F32 || d == WQ_BF16 || d == WQ_F16; }

int check_packed(wq_ctx* ctx, const wq_packed_kv* kv, int B, bool need_tables)
{
    if (!kv) return wq_fail(ctx, WQ_ERR_ARG, "packed cache descriptor is NULL");
    if (kv->B != B) return wq_fail(ctx, WQ_ERR_ARG, "packed cache is for B=%d, call has B=%d", kv->B, B);
    if (!shape_ok(kv->Hkv, kv->hd, kv->group))
        return wq_fail(ctx, WQ_ERR_UNSUPPORTED, "unsupported shape Hkv=%d hd=%d group=%d", kv->Hkv, kv->hd, kv->group);
    if (kv->dtype16 != WQ_BF16 && kv->dtype16 != WQ_F16)
        return wq_fail(ctx, WQ_ERR_ARG, "dtype16 must be WQ_BF16 or WQ_F16");
    for (int c = 0; c < 3; c++) {
        if (kv->cap[c] < 0 || kv->cap[c] % 32 != 0)
            return wq_fail(ctx, WQ_ERR_ARG, "cap[%d]=%lld is not a non-negative multiple of 32", c, (long long)kv->cap[c]);
        if (kv->cap[c] > (int64_t)1 << 26) return wq_fail(ctx, WQ_ERR_UNSUPPORTED, "cap[%d] above 2^26 tokens", c);
        if (kv->cap[c] > 0 && (!kv->codes[c] || !kv->meta[c]))
            return wq_fail(ctx, WQ_ERR_ARG, "class %d has capacity but NULL codes/meta", c);
        if (need_tables && (!kv->cls_off[c] || !kv->cls_len[c]))
            return wq_fail(ctx, WQ_ERR_ARG, "class %d offset/length tables are NULL", c);
    }
    if (kv->cap16 < 0 || kv->cap16 > (int64_t)1 << 26) return wq_fail(ctx, WQ_ERR_ARG, "bad cap16");
    if (kv->cap16 > 0 && (!kv->k16 || !kv->v16)) return wq_fail(ctx, WQ_ERR_ARG, "16-bit segment has capacity but NULL k16/v16");
    if (!kv->off16 || !kv->len16) return wq_fail(ctx, WQ_ERR_ARG, "off16/len16 tables are NULL");
    if (!kv->v_scale_max) return wq_fail(ctx, WQ_ERR_ARG, "v_scale_max table is NULL");
    return WQ_OK;
}

}  // namespace

extern "C" {

int wq_create(wq_ctx** out, void* hip_stream, void* workspace, size_t workspace_bytes)
{
    if (!out) return WQ_ERR_ARG;
    *out = nullptr;
    wq_ctx* ctx = new (std::nothrow) wq_ctx();
    if (!ctx) return WQ_ERR_ARG;
    ctx->stream = static_cast<hipStream_t>(hip_stream);
    ctx->ws = static_cast<char*>(workspace);
    ctx->ws_bytes = workspace_bytes;
    ctx->owns_ws = false;
    ctx->timing = false;
    for (int i = 0; i < 2 * WQ_TIMING_RING; i++) ctx->ev[i] = nullptr;
    ctx->ev_calls = 0;
    ctx->err[0] = 0;
    if (!workspace && workspace_bytes > 0) {
        void* p = nullptr;
        if (hipMalloc(&p, workspace_bytes) != hipSuccess) {
            delete ctx;
            return WQ_ERR_HIP;
        }
        ctx->ws = static_cast<char*>(p);
        ctx->owns_ws = true;
    }
    if (ctx->ws && ctx->ws_bytes >= WQ_WS_HEADER && ctx->owns_ws) {
        if (hipMemset(ctx->ws, 0, WQ_WS_HEADER) != hipSuccess) {
            (void)hipFree(ctx->ws);
            delete ctx;
            return WQ_ERR_HIP;
        }
    }
    *out = ctx;
    return WQ_OK;
}

int wq_destroy(wq_ctx* ctx)
{
    if (!ctx) return WQ_OK;
    if (ctx->owns_ws && ctx->ws) (void)hipFree(ctx->ws);
    for (int i = 0; i < 2 * WQ_TIMING_RING; i++)
        if (ctx->ev[i]) (void)hipEventDestroy(ctx->ev[i]);
    delete ctx;
    return WQ_OK;
}

int wq_set_stream(wq_ctx* ctx, void* hip_stream)
{
    if (!ctx) return WQ_ERR_ARG;
    ctx->stream = static_cast<hipStream_t>(hip_stream);
    return WQ_OK;
}

const char* wq_last_error(const wq_ctx* ctx) { return ctx ? ctx->err : "null context"; }

int wq_device_status(wq_ctx* ctx, uint32_t* bits)
{
    if (!ctx || !bits) return WQ_ERR_ARG;
    if (!ctx->ws || ctx->ws_bytes < WQ_WS_HEADER) return wq_fail(ctx, WQ_ERR_WORKSPACE, "no workspace");
    WQ_HIP_CHECK(ctx, hipMemcpyAsync(bits, ctx->ws, sizeof(uint32_t), hipMemcpyDeviceToHost, ctx->stream));
    WQ_HIP_CHECK(ctx, hipStreamSynchronize(ctx->stream));
    WQ_HIP_CHECK(ctx, hipMemsetAsync(ctx->ws, 0, sizeof(uint32_t), ctx->stream));
    return WQ_OK;
}

size_t wq_workspace_bytes(int B, int Hq, int hd, int max_splits, int64_t total_vis, int64_t total_txt, int D)
{
    size_t a = wq_decode_ws_bytes(B, Hq, hd, max_splits);
    size_t b = wq_scores_ws_bytes(B, total_vis, total_txt, D);
    size_t c = wq_align256(sizeof(int32_t) * (size_t)(B > 0 ? B + 1 : 1));   // prefix of 16-bit rows (a3)
    size_t m = a > b ? a : b;
    if (c > m) m = c;
    return WQ_WS_HEADER + m;
}

size_t wq_v_scale_floats(int B, int Hkv, const int64_t cap[3])
{
    if (B < 0 || Hkv <= 0 || !cap) return 0;
    size_t blocks = 0;
    for (int c = 0; c < 3; c++) blocks += (size_t)((cap[c] > 0 ? cap[c] : 0) / 32);
    return (size_t)B + blocks * (size_t)Hkv;
}

size_t wq_packed_bytes(int bits, int64_t cap_tokens, int Hkv, int hd, int group, size_t* meta_bytes)
{
    if (meta_bytes) *meta_bytes = 0;
    if (!(bits == 2 || bits == 4 || bits == 8) || cap_tokens < 0 || !shape_ok(Hkv, hd, group)) return 0;
    int64_t cap = (cap_tokens + 31) / 32 * 32;
    if (meta_bytes) *meta_bytes = (size_t)2 * Hkv * cap * (hd / group) * 4;
    return (size_t)2 * Hkv * cap * hd * bits / 8;
}

// total_tokens well below B * max_seq_tokens: the sequences differ in length, and the launch gives a sequence splits in
// proportion to its length (the longest gets them all): more splits, so that about as many workgroups as for equal
// lengths have work
int wq_auto_splits_ragged(int B, int Hkv, int64_t max_seq_tokens, int64_t total_tokens)
{
    const int s0 = wq_auto_splits(B, Hkv, max_seq_tokens);
    if (B <= 0 || max_seq_tokens <= 0 || total_tokens <= 0) return s0;
    const double fill = (double)total_tokens / ((double)B * (double)max_seq_tokens);
    if (fill >= 0.75) return s0;
    // twice the count that would give as many busy workgroups as equal lengths do: with lengths this uneven the launch is as
    // long as its longest sequences take, and more, smaller workgroups on them end earlier (measured on 32 sequences of
    // 8 to 128 frames: 84.7 us with 2 splits for all, 77.4 with 4 by length, 72.5 with 8 by length, 82.6 with 12)
    int64_t s = (int64_t)(2.0 * (double)s0 / fill + 0.5);
    const int64_t most = (max_seq_tokens + 1023) / 1024;
    if (s > most) s = most;
    if (s > 256) s = 256;
    return s > s0 ? (int)s : s0;
}

int wq_auto_splits(int B, int Hkv, int64_t max_seq_tokens)
{
    if (B <= 0 || Hkv <= 0) return 1;
    // one workgroup of eight wavefronts per compute unit (256 CUs) is what the decode kernel's registers allow;
    // more splits only add per-workgroup set-up.  Keep at least 1024 tokens per workgroup.
    int64_t want = (256 + (int64_t)B * Hkv - 1) / ((int64_t)B * Hkv);
    int64_t most = max_seq_tokens > 0 ? (max_seq_tokens + 1023) / 1024 : 1;
    if (want > most) want = most;
    if (want < 1) want = 1;
    if (want > 256) want = 256;
    return (int)want;
}

int wq_window_scores(wq_ctx* ctx, const void* vis_emb, const void* txt_emb, int dtype, int B, int D,
                     const int32_t* vis_off, const int32_t* txt_off, const int32_t* win_size, const int32_t* win_off,
                     int64_t total_vis, int64_t total_txt, int64_t total_win, int algo, float* scores)
{
    if (!ctx) return WQ_ERR_ARG;
    if (B < 0 || D <= 0 || total_vis < 0 || total_txt < 0 || total_win < 0)
        return wq_fail(ctx, WQ_ERR_ARG, "negative size (B=%d D=%d)", B, D);
    if (!dtype_ok(dtype)) return wq_fail(ctx, WQ_ERR_ARG, "unknown dtype %d", dtype);
    if (algo != WQ_SCORE_AUTO && algo != WQ_SCORE_PAIRWISE_MFMA && algo != WQ_SCORE_POOLED)
        return wq_fail(ctx, WQ_ERR_ARG, "unknown scoring algorithm %d", algo);
    if (total_vis > INT32_MAX || total_txt > INT32_MAX) return wq_fail(ctx, WQ_ERR_UNSUPPORTED, "too many rows");
    if (B == 0 || total_win == 0) return WQ_OK;
    if (!vis_off || !txt_off || !win_size || !win_off || !scores) return wq_fail(ctx, WQ_ERR_ARG, "NULL table or output");
    if ((total_vis > 0 && !vis_emb) || (total_txt > 0 && !txt_emb)) return wq_fail(ctx, WQ_ERR_ARG, "NULL embeddings");
    if (algo == WQ_SCORE_PAIRWISE_MFMA && dtype == WQ_F32)
        return wq_fail(ctx, WQ_ERR_UNSUPPORTED, "the matrix-core scoring path takes bf16 or fp16 embeddings");
    if (algo == WQ_SCORE_PAIRWISE_MFMA && D % 128 != 0)
        return wq_fail(ctx, WQ_ERR_UNSUPPORTED, "the matrix-core scoring path needs D %% 128 == 0");
    if (ctx->ws_bytes < WQ_WS_HEADER + wq_scores_ws_bytes(B, total_vis, total_txt, D))
        return wq_fail(ctx, WQ_ERR_WORKSPACE, "workspace too small for scoring");
    return wq_launch_scores(ctx, vis_emb, txt_emb, dtype, B, D, vis_off, txt_off, win_size, win_off, total_vis,
                            total_txt, total_win, algo, scores);
}

int wq_assign_bits(wq_ctx* ctx, const float* scores, int B, const int32_t* win_off, int max_windows, int mode,
                   const int32_t* quota, const float* thresholds, int top_bits, int pin_first, uint8_t* bits,
                   int32_t* perm, int32_t* seg_windows)
{
    if (!ctx) return WQ_ERR_ARG;
    if (B < 0 || max_windows < 0) return wq_fail(ctx, WQ_ERR_ARG, "negative size");
    if (mode != WQ_MODE_QUOTA && mode != WQ_MODE_THRESHOLD) return wq_fail(ctx, WQ_ERR_ARG, "unknown mode %d", mode);
    if (top_bits != 8 && top_bits != 16) return wq_fail(ctx, WQ_ERR_ARG, "top_bits must be 8 or 16, got %d", top_bits);
    if (max_windows > WQ_MAX_WINDOWS)
        return wq_fail(ctx, WQ_ERR_UNSUPPORTED, "more than %d windows per sequence", WQ_MAX_WINDOWS);
    if (B == 0) return WQ_OK;
    if (!win_off || !seg_windows) return wq_fail(ctx, WQ_ERR_ARG, "NULL table");
    if (max_windows > 0 && (!scores || !bits || !perm)) return wq_fail(ctx, WQ_ERR_ARG, "NULL scores or output");
    if (mode == WQ_MODE_QUOTA && !quota) return wq_fail(ctx, WQ_ERR_ARG, "quota mode without quota table");
    if (mode == WQ_MODE_THRESHOLD && !thresholds) return wq_fail(ctx, WQ_ERR_ARG, "threshold mode without thresholds");
    if (!ctx->ws || ctx->ws_bytes < WQ_WS_HEADER) return wq_fail(ctx, WQ_ERR_WORKSPACE, "no workspace");
    return wq_launch_assign(ctx, scores, B, win_off, max_windows, mode, quota, thresholds, top_bits, pin_first != 0,
                            bits, perm, seg_windows);
}

int wq_layer_thresholds(const double* s, int n_layers, double alpha, float* t_low, float* t_high)
{
    if (n_layers < 0 || !isfinite(alpha)) return WQ_ERR_ARG;
    if (n_layers > 0 && (!s || !t_low || !t_high)) return WQ_ERR_ARG;
    for (int i = 0; i < n_layers; i++)
        if (!(s[i] >= 0.0 && s[i] <= 1.0)) return WQ_ERR_ARG;
    for (int i = 0; i < n_layers; i++) {
        // expm1 keeps the quotient accurate where alpha * s is small; alpha = 0 is the limit s
        const double lo = alpha == 0.0 ? s[i] : expm1(alpha * s[i]) / expm1(alpha);
        const double hi = alpha == 0.0 ? s[i] : expm1(-alpha * s[i]) / expm1(-alpha);
        t_low[i] = (float)lo;
        t_high[i] = (float)hi;
    }
    return WQ_OK;
}

int wq_vote_bits(wq_ctx* ctx, const uint8_t* bits_in, int B, const int32_t* win_off, int max_windows, uint8_t* bits_out,
                 int32_t* perm, int32_t* seg_windows)
{
    if (!ctx) return WQ_ERR_ARG;
    if (B < 0 || max_windows < 0) return wq_fail(ctx, WQ_ERR_ARG, "negative size");
    if (max_windows > WQ_MAX_WINDOWS)
        return wq_fail(ctx, WQ_ERR_UNSUPPORTED, "more than %d windows per sequence", WQ_MAX_WINDOWS);
    if (B == 0) return WQ_OK;
    if (!win_off || !seg_windows) return wq_fail(ctx, WQ_ERR_ARG, "NULL table");
    if (max_windows > 0 && (!bits_in || !bits_out || !perm)) return wq_fail(ctx, WQ_ERR_ARG, "NULL widths or output");
    if (!ctx->ws || ctx->ws_bytes < WQ_WS_HEADER) return wq_fail(ctx, WQ_ERR_WORKSPACE, "no workspace");
    return wq_launch_vote(ctx, bits_in, B, win_off, max_windows, bits_out, perm, seg_windows);
}

int wq_validate_assignment(wq_ctx* ctx, int B, const int32_t* win_off, int max_windows, const int32_t* perm, const int32_t* seg_windows)
{
    if (!ctx) return WQ_ERR_ARG;
    if (B < 0 || max_windows < 0) return wq_fail(ctx, WQ_ERR_ARG, "negative size");
    if (max_windows > WQ_MAX_WINDOWS)
        return wq_fail(ctx, WQ_ERR_UNSUPPORTED, "more than %d windows per sequence", WQ_MAX_WINDOWS);
    if (B == 0) return WQ_OK;
    if (!win_off || !seg_windows || (max_windows > 0 && !perm)) return wq_fail(ctx, WQ_ERR_ARG, "NULL table");
    if (!ctx->ws || ctx->ws_bytes < WQ_WS_HEADER) return wq_fail(ctx, WQ_ERR_WORKSPACE, "no workspace");
    return wq_launch_validate(ctx, B, win_off, max_windows, perm, seg_windows);
}

int wq_reorder_quantize(wq_ctx* ctx, const void* K, const void* V, int dtype, int B, const int32_t* kv_off,
                        const int32_t* win_size, const int32_t* win_off, const int32_t* perm,
                        const int32_t* seg_windows, int64_t total_rows, const wq_packed_kv* out)
{
    if (!ctx) return WQ_ERR_ARG;
    if (B < 0 || total_rows < 0) return wq_fail(ctx, WQ_ERR_ARG, "negative size");
    if (!dtype_ok(dtype)) return wq_fail(ctx, WQ_ERR_ARG, "unknown dtype %d", dtype);
    int rc = check_packed(ctx, out, B, true);
    if (rc != WQ_OK) return rc;
    if ((dtype == WQ_BF16) != (out->dtype16 == WQ_BF16))
        return wq_fail(ctx, WQ_ERR_ARG, "dtype16 must be bf16 for bf16 input and fp16 for fp16/fp32 input");
    if (total_rows > INT32_MAX) return wq_fail(ctx, WQ_ERR_UNSUPPORTED, "too many rows");
    if (B == 0) return WQ_OK;
    if (!kv_off || !win_size || !win_off || !seg_windows) return wq_fail(ctx, WQ_ERR_ARG, "NULL table");
    if (total_rows > 0 && (!K || !V || !perm)) return wq_fail(ctx, WQ_ERR_ARG, "NULL K, V or perm");
    if ((reinterpret_cast<uintptr_t>(K) | reinterpret_cast<uintptr_t>(V)) % 16 != 0)
        return wq_fail(ctx, WQ_ERR_ARG, "K and V must be 16-byte aligned");
    if (ctx->ws_bytes < WQ_WS_HEADER + wq_align256(sizeof(int32_t) * (size_t)(B + 1)))
        return wq_fail(ctx, WQ_ERR_WORKSPACE, "workspace too small for reorder_quantize");
    return wq_launch_quantize(ctx, K, V, dtype, B, kv_off, win_size, win_off, perm, seg_windows, total_rows, out);
}

int wq_append_kv(wq_ctx* ctx, const void* k_new, const void* v_new, int dtype, int B, const wq_packed_kv* kv)
{
    if (!ctx) return WQ_ERR_ARG;
    if (B < 0) return wq_fail(ctx, WQ_ERR_ARG, "negative size");
    if (!dtype_ok(dtype)) return wq_fail(ctx, WQ_ERR_ARG, "unknown dtype %d", dtype);
    int rc = check_packed(ctx, kv, B, false);
    if (rc != WQ_OK) return rc;
    if ((dtype == WQ_BF16) != (kv->dtype16 == WQ_BF16))
        return wq_fail(ctx, WQ_ERR_ARG, "dtype16 must be bf16 for bf16 input and fp16 for fp16/fp32 input");
    if (B == 0) return WQ_OK;
    if (!k_new || !v_new) return wq_fail(ctx, WQ_ERR_ARG, "NULL k_new or v_new");
    if (!ctx->ws || ctx->ws_bytes < WQ_WS_HEADER) return wq_fail(ctx, WQ_ERR_WORKSPACE, "no workspace");
    return wq_launch_append(ctx, k_new, v_new, dtype, B, kv);
}

// What both decode entry points check before anything is enqueued; resolves num_splits == 0.
static int check_decode(wq_ctx* ctx, const void* q, int q_dtype, int B, int Hq, const wq_packed_kv* kv, float sm_scale,
                        int* num_splits, int64_t max_seq_tokens, int algo, const float* out, int64_t* longest)
{
    *longest = 0;
    if (B < 0 || Hq <= 0) return wq_fail(ctx, WQ_ERR_ARG, "bad B or Hq");
    if (B > 65535) return wq_fail(ctx, WQ_ERR_UNSUPPORTED, "more than 65535 sequences in one call");      // a grid dimension
    if (!dtype_ok(q_dtype)) return wq_fail(ctx, WQ_ERR_ARG, "unknown q dtype %d", q_dtype);
    int rc = check_packed(ctx, kv, B, true);
    if (rc != WQ_OK) return rc;
    if (Hq % kv->Hkv != 0 || Hq / kv->Hkv > WQ_MAX_REP)
        return wq_fail(ctx, WQ_ERR_UNSUPPORTED, "Hq=%d must be a multiple of Hkv=%d, at most %d query heads per KV head",
                       Hq, kv->Hkv, WQ_MAX_REP);
    const int balgo = algo & ~WQ_DECODE_FLAGS;
    const bool by_length = (algo & WQ_DECODE_BY_LENGTH) != 0;
    if (by_length && max_seq_tokens <= 0) return wq_fail(ctx, WQ_ERR_ARG, "WQ_DECODE_BY_LENGTH needs max_seq_tokens");
    if (balgo != WQ_DECODE_AUTO && balgo != WQ_DECODE_GENERIC && balgo != WQ_DECODE_MFMA)
        return wq_fail(ctx, WQ_ERR_ARG, "unknown decode algorithm %d", algo);
    if (balgo == WQ_DECODE_MFMA && kv->hd / kv->group != 2)
        return wq_fail(ctx, WQ_ERR_UNSUPPORTED, "the matrix-core decode kernel needs hd/group == 2");
    if (*num_splits < 0 || *num_splits > 1024) return wq_fail(ctx, WQ_ERR_ARG, "num_splits out of range");
    if (!(sm_scale > 0.0f) || sm_scale > 3.0e38f) return wq_fail(ctx, WQ_ERR_ARG, "sm_scale must be positive and finite");
    if (B == 0) return WQ_OK;
    if (!q || !out) return wq_fail(ctx, WQ_ERR_ARG, "NULL q or out");
    if (by_length) *longest = max_seq_tokens;
    if (*num_splits == 0) {
        *num_splits = wq_auto_splits(B, kv->Hkv, max_seq_tokens);
        if (by_length) {    // more splits (the caches' capacities stand in for the tokens), if the workspace has room for them
            int more = wq_auto_splits_ragged(B, kv->Hkv, max_seq_tokens, kv->cap[0] + kv->cap[1] + kv->cap[2] + kv->cap16);
            if (more > WQ_MAX_FUSED_SPLITS) more = WQ_MAX_FUSED_SPLITS;    // (splits by length need the merge inside the kernel)
            if (more > *num_splits && ctx->ws_bytes >= WQ_WS_HEADER + wq_decode_ws_bytes(B, Hq, kv->hd, more)) *num_splits = more;
        }
    }
    if (ctx->ws_bytes < WQ_WS_HEADER + wq_decode_ws_bytes(B, Hq, kv->hd, *num_splits))
        return wq_fail(ctx, WQ_ERR_WORKSPACE, "workspace too small for %d splits", *num_splits);
    return WQ_OK;
}

int wq_decode_append_attention(wq_ctx* ctx, const void* q, int q_dtype, int B, int Hq, const wq_packed_kv* kv,
                               const void* k_new, const void* v_new, int new_dtype, float sm_scale, int num_splits,
                               int64_t max_seq_tokens, int algo, float* out, float* lse)
{
    if (!ctx) return WQ_ERR_ARG;
    if (!dtype_ok(new_dtype)) return wq_fail(ctx, WQ_ERR_ARG, "unknown dtype %d", new_dtype);
    if (kv && (new_dtype == WQ_BF16) != (kv->dtype16 == WQ_BF16))
        return wq_fail(ctx, WQ_ERR_ARG, "dtype16 must be bf16 for bf16 input and fp16 for fp16/fp32 input");
    if (B > 0 && (!k_new || !v_new)) return wq_fail(ctx, WQ_ERR_ARG, "NULL k_new or v_new");
    if (algo & WQ_DECODE_PARTIALS_ONLY) return wq_fail(ctx, WQ_ERR_ARG, "partials-only launches do not append");
    int64_t longest = 0;
    int rc = check_decode(ctx, q, q_dtype, B, Hq, kv, sm_scale, &num_splits, max_seq_tokens, algo, out, &longest);
    if (rc != WQ_OK || B == 0) return rc;
    if (wq_decode_can_append(q_dtype, B, Hq, kv, num_splits, algo, new_dtype))
        return wq_launch_decode(ctx, q, q_dtype, B, Hq, kv, sm_scale, num_splits, algo, out, lse, k_new, v_new, longest);
    // other kernels, other element types: two launches
    rc = wq_launch_append(ctx, k_new, v_new, new_dtype, B, kv);
    if (rc != WQ_OK) return rc;
    return wq_launch_decode(ctx, q, q_dtype, B, Hq, kv, sm_scale, num_splits, algo, out, lse, nullptr, nullptr, longest);
}

int wq_dequantize(wq_ctx* ctx, int B, const wq_packed_kv* src, const wq_packed_kv* dst)
{
    if (!ctx) return WQ_ERR_ARG;
    if (B < 0) return wq_fail(ctx, WQ_ERR_ARG, "negative size");
    int rc = check_packed(ctx, src, B, true);
    if (rc != WQ_OK) return rc;
    rc = check_packed(ctx, dst, B, true);
    if (rc != WQ_OK) return rc;
    if (src->Hkv != dst->Hkv || src->hd != dst->hd || src->dtype16 != dst->dtype16)
        return wq_fail(ctx, WQ_ERR_ARG, "source and destination differ in Hkv, hd or dtype16");
    if (src->k16 == dst->k16 || src->v16 == dst->v16) return wq_fail(ctx, WQ_ERR_ARG, "source and destination share their 16-bit segment");
    if (B == 0) return WQ_OK;
    if (!ctx->ws || ctx->ws_bytes < WQ_WS_HEADER) return wq_fail(ctx, WQ_ERR_WORKSPACE, "no workspace");
    return wq_launch_dequantize(ctx, B, src, dst);
}

int wq_decode_attention(wq_ctx* ctx, const void* q, int q_dtype, int B, int Hq, const wq_packed_kv* kv,
                        float sm_scale, int num_splits, int64_t max_seq_tokens, int algo, float* out, float* lse)
{
    if (!ctx) return WQ_ERR_ARG;
    int64_t longest = 0;
    const int rc = check_decode(ctx, q, q_dtype, B, Hq, kv, sm_scale, &num_splits, max_seq_tokens, algo, out, &longest);
    if (rc != WQ_OK || B == 0) return rc;
    return wq_launch_decode(ctx, q, q_dtype, B, Hq, kv, sm_scale, num_splits, algo, out, lse, nullptr, nullptr, longest);
}

// ---- the entry point that allocates nothing ---------------------------------------------------------------------
// Its workspace is this array, part of the code object: every GPU that loads the library holds its own copy at its own
// address.  The name is a host-side stand-in for the symbol; the device address comes from hipGetSymbolAddress, once per
// device, and only that address is handed to kernels.  Zero-initialised when the code object is loaded, which is the
// state a workspace header has to start in.
static __device__ __align__(256) unsigned char scratch[WQ_STATIC_SCRATCH_BYTES];

namespace {
constexpr int WQ_MAX_DEVICES = 64;
struct StaticSlot {
    bool ready = false;
    wq_ctx ctx;
};
StaticSlot g_static[WQ_MAX_DEVICES];
std::mutex g_static_mu;
char g_static_err[256] = "";
}  // namespace

const char* wq_static_last_error(void)
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= WQ_MAX_DEVICES) return g_static_err;
    return g_static[dev].ready ? g_static[dev].ctx.err : g_static_err;
}

int wq_decode_attention_static(void* hip_stream, const void* q, int q_dtype, int B, int Hq, const wq_packed_kv* kv,
                               float sm_scale, int num_splits, int64_t max_seq_tokens, int algo, float* out, float* lse)
{
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess || dev < 0 || dev >= WQ_MAX_DEVICES) {
        snprintf(g_static_err, sizeof(g_static_err), "no current device (%s)", e != hipSuccess ? hipGetErrorString(e) : "index out of range");
        return WQ_ERR_HIP;
    }
    StaticSlot& slot = g_static[dev];
    {
        std::lock_guard<std::mutex> lock(g_static_mu);
        if (!slot.ready) {
            void* ptr = nullptr;
            e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
            if (e != hipSuccess || !ptr) {
                snprintf(g_static_err, sizeof(g_static_err), "hipGetSymbolAddress(scratch): %s", hipGetErrorString(e));
                return WQ_ERR_HIP;
            }
            slot.ctx.stream = nullptr;
            slot.ctx.ws = static_cast<char*>(ptr);
            slot.ctx.ws_bytes = WQ_STATIC_SCRATCH_BYTES;
            slot.ctx.owns_ws = false;
            slot.ctx.timing = false;
            for (int i = 0; i < 2 * WQ_TIMING_RING; i++) slot.ctx.ev[i] = nullptr;
            slot.ctx.ev_calls = 0;
            slot.ctx.err[0] = 0;
            slot.ready = true;
        }
    }
    wq_ctx* ctx = &slot.ctx;
    ctx->stream = static_cast<hipStream_t>(hip_stream);
    int64_t longest = 0;
    int splits = num_splits;
    const int rc = check_decode(ctx, q, q_dtype, B, Hq, kv, sm_scale, &splits, max_seq_tokens, algo, out, &longest);
    if (rc == WQ_ERR_WORKSPACE)
        return wq_fail(ctx, WQ_ERR_WORKSPACE, "B=%d Hq=%d hd=%d with %d splits needs %zu bytes of scratch, the static array holds %u", B, Hq,
                       kv->hd, splits, WQ_WS_HEADER + wq_decode_ws_bytes(B, Hq, kv->hd, splits), (unsigned)WQ_STATIC_SCRATCH_BYTES);
    if (rc != WQ_OK || B == 0) return rc;
    return wq_launch_decode(ctx, q, q_dtype, B, Hq, kv, sm_scale, splits, algo, out, lse, nullptr, nullptr, longest);
}

}  // extern "C"
