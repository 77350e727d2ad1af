// Measurement aids of libwq (include/wq_measure.h): plain streaming and matrix-core probes, and the event ring that times
// the decode kernel.  Nothing here is part of the method; the four calls of wq.h do not depend on it.
#include "wq_internal.h"
#include "../../include/wq_measure.h"

extern "C" {

int wq_decode_timing(wq_ctx* ctx, int enable)
{
    if (!ctx) return WQ_ERR_ARG;
    if (enable && !ctx->ev[0])
        for (int i = 0; i < 2 * WQ_TIMING_RING; i++) WQ_HIP_CHECK(ctx, hipEventCreate(&ctx->ev[i]));
    ctx->timing = enable != 0;
    ctx->ev_calls = 0;
    return WQ_OK;
}

int wq_decode_times_us(wq_ctx* ctx, float* us, int n)
{
    if (!ctx || !us || n < 0 || !ctx->ev[0]) return WQ_ERR_ARG;
    if ((uint64_t)n > ctx->ev_calls || n > WQ_TIMING_RING) return wq_fail(ctx, WQ_ERR_ARG, "only %llu timed calls, ring of %d",
                                                                          (unsigned long long)ctx->ev_calls, WQ_TIMING_RING);
    for (int k = 0; k < n; k++) {                    // oldest of the last n first
        const uint64_t call = ctx->ev_calls - (uint64_t)n + (uint64_t)k;
        const int slot = (int)(call % WQ_TIMING_RING);
        float ms = 0.f;
        WQ_HIP_CHECK(ctx, hipEventSynchronize(ctx->ev[2 * slot + 1]));
        WQ_HIP_CHECK(ctx, hipEventElapsedTime(&ms, ctx->ev[2 * slot], ctx->ev[2 * slot + 1]));
        us[k] = ms * 1000.0f;
    }
    return WQ_OK;
}

}  // extern "C"

namespace {
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
}  // namespace

// ---- plain streaming kernels of known size -----------------------
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

namespace {

__device__ __forceinline__ uint32_t probe_mix(uint32_t x)
{
    x ^= x >> 16; x *= 0x7feb352du; x ^= x >> 15; x *= 0x846ca68bu; x ^= x >> 16;
    return x;
}

// 32 independent accumulator tiles per wavefront, operands in registers only; RANDOM: bf16 values in (-2, 2), 8 x 4
// different operand pairs in a row, moved to other products every 128 products; else all ones.
template <bool RANDOM>
__global__ __launch_bounds__(512) void k_probe_mfma(uint32_t* __restrict__ sink, int iters)
{
    floatx4s acc[32];
#pragma unroll
    for (int i = 0; i < 32; i++) acc[i] = floatx4s{0.f, 0.f, 0.f, 0.f};
    uint32_t s = probe_mix(blockIdx.x * 512 + threadIdx.x + 1);
    auto rnd = [&]() { s = probe_mix(s + 0x9e3779b9u); return RANDOM ? ((s & 0x80ff80ffu) | 0x3f003f00u) : 0x3f803f80u; };
    uint4 a[8], b[4];
#pragma unroll
    for (int i = 0; i < 8; i++) a[i] = make_uint4(rnd(), rnd(), rnd(), rnd());
#pragma unroll
    for (int i = 0; i < 4; i++) b[i] = make_uint4(rnd(), rnd(), rnd(), rnd());
    for (int it = 0; it < iters; it += 4) {         // iters is a multiple of 4 (checked by the host)
#pragma unroll
        for (int r = 0; r < 4; r++)
#pragma unroll
            for (int i = 0; i < 8; i++)
#pragma unroll
                for (int j = 0; j < 4; j++) acc[i * 4 + j] = mfma_s<true>(a[i], b[j], acc[i * 4 + j]);
        if (RANDOM) {                               // 48 register moves per 128 products
            const uint4 t = a[0];
#pragma unroll
            for (int i = 0; i < 7; i++) a[i] = a[i + 1];
            a[7] = make_uint4(t.y, t.z, t.w, t.x);
            const uint4 u = b[0];
            b[0] = b[1], b[1] = b[2], b[2] = b[3], b[3] = make_uint4(u.w, u.x, u.y, u.z);
        }
    }
    float r = 0.f;
#pragma unroll
    for (int i = 0; i < 32; i++) r += acc[i][0] + acc[i][1] + acc[i][2] + acc[i][3];
    if (__float_as_uint(r) == 0x9E3779B9u) sink[0] = 1u;   // practically never true; keeps the products alive
}

}  // namespace

extern "C" int wq_probe_mfma(wq_ctx* ctx, int random_operands, int workgroups, int iters, double* flops)
{
    if (!ctx || workgroups <= 0 || iters <= 0 || iters % 4 != 0) return WQ_ERR_ARG;
    if (!ctx->ws || ctx->ws_bytes < WQ_WS_HEADER) return wq_fail(ctx, WQ_ERR_WORKSPACE, "no workspace");
    if (random_operands)
        hipLaunchKernelGGL(k_probe_mfma<true>, dim3(workgroups), dim3(512), 0, ctx->stream, wq_status_ptr(ctx) + 8, iters);
    else
        hipLaunchKernelGGL(k_probe_mfma<false>, dim3(workgroups), dim3(512), 0, ctx->stream, wq_status_ptr(ctx) + 8, iters);
    WQ_HIP_CHECK(ctx, hipGetLastError());
    if (flops) *flops = (double)workgroups * 8.0 * (double)iters * 32.0 * (2.0 * 16 * 16 * 32);
    return WQ_OK;
}

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
