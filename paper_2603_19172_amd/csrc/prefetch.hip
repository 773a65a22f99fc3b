// Host-resident experts: copies from pinned host memory into device buffers on
// a side stream, handed over to the compute stream through events, and the
// residual + normalisation step that chains layers of a stack.
#include <math.h>

#include "common.hpp"

namespace dymoe {

// v = h[t,:] + alpha * y[t,:];  h_out[t,:] = bf16(v / rms(v)), fp32 arithmetic.  One workgroup per token: a thread
// takes 8 consecutive elements at a time (16-byte loads; VEC = false: one element at a time, for row lengths or
// pointers that rule those out), the squares are summed per thread, per wavefront, then over the wavefronts in order.
constexpr int kNormThreads = 256;

template <typename YT, bool VEC>
__global__ __launch_bounds__(kNormThreads) void residual_rmsnorm_kernel(const uint16_t* __restrict__ h,
                                                                       const YT* __restrict__ y, float alpha,
                                                                       int T, int H, uint16_t* __restrict__ out)
{
    __shared__ float s_part[kNormThreads / kWave];
    const int t = blockIdx.x;
    const uint16_t* hr = h + (size_t)t * H;
    const YT* yr = y + (size_t)t * H;
    uint16_t* orow = out + (size_t)t * H;
    constexpr int W = VEC ? 8 : 1;
    auto value = [&](int j, float (&v)[W]) {
        if constexpr (VEC) {
            float hv[8], yv[8];
            const uint4 hraw = *reinterpret_cast<const uint4*>(hr + j);
            hv[0] = bf16_lo(hraw.x); hv[1] = bf16_hi(hraw.x); hv[2] = bf16_lo(hraw.y); hv[3] = bf16_hi(hraw.y);
            hv[4] = bf16_lo(hraw.z); hv[5] = bf16_hi(hraw.z); hv[6] = bf16_lo(hraw.w); hv[7] = bf16_hi(hraw.w);
            if constexpr (sizeof(YT) == 2) {
                const uint4 yraw = *reinterpret_cast<const uint4*>(yr + j);
                yv[0] = bf16_lo(yraw.x); yv[1] = bf16_hi(yraw.x); yv[2] = bf16_lo(yraw.y); yv[3] = bf16_hi(yraw.y);
                yv[4] = bf16_lo(yraw.z); yv[5] = bf16_hi(yraw.z); yv[6] = bf16_lo(yraw.w); yv[7] = bf16_hi(yraw.w);
            } else {
                const float4 a = *reinterpret_cast<const float4*>(yr + j);
                const float4 b = *reinterpret_cast<const float4*>(yr + j + 4);
                yv[0] = a.x; yv[1] = a.y; yv[2] = a.z; yv[3] = a.w; yv[4] = b.x; yv[5] = b.y; yv[6] = b.z; yv[7] = b.w;
            }
#pragma unroll
            for (int i = 0; i < 8; i++) v[i] = fmaf(alpha, yv[i], hv[i]);
        } else {
            float yv;
            if constexpr (sizeof(YT) == 2) yv = bf16_bits_to_f32(yr[j]);
            else yv = yr[j];
            v[0] = fmaf(alpha, yv, bf16_bits_to_f32(hr[j]));
        }
    };
    float ss = 0.0f;
    for (int j = threadIdx.x * W; j < H; j += kNormThreads * W) {
        float v[W];
        value(j, v);
#pragma unroll
        for (int i = 0; i < W; i++) ss = fmaf(v[i], v[i], ss);
    }
    ss = wave_sum(ss);
    if ((threadIdx.x & (kWave - 1)) == 0) s_part[threadIdx.x / kWave] = ss;
    __syncthreads();
    float tot = 0.0f;
#pragma unroll
    for (int wv = 0; wv < kNormThreads / kWave; wv++) tot += s_part[wv];
    const float inv = (tot > 0.0f) ? 1.0f / sqrtf(tot / (float)H) : 0.0f;
    for (int j = threadIdx.x * W; j < H; j += kNormThreads * W) {
        float v[W];
        value(j, v);
        if constexpr (VEC) {
            uint4 o;
            o.x = f32_to_bf16_bits(v[0] * inv) | (f32_to_bf16_bits(v[1] * inv) << 16);
            o.y = f32_to_bf16_bits(v[2] * inv) | (f32_to_bf16_bits(v[3] * inv) << 16);
            o.z = f32_to_bf16_bits(v[4] * inv) | (f32_to_bf16_bits(v[5] * inv) << 16);
            o.w = f32_to_bf16_bits(v[6] * inv) | (f32_to_bf16_bits(v[7] * inv) << 16);
            *reinterpret_cast<uint4*>(orow + j) = o;
        } else {
            orow[j] = (uint16_t)f32_to_bf16_bits(v[0] * inv);
        }
    }
}

}  // namespace dymoe

extern "C" {

int dymoe_prefetch_submit(dymoe_ctx* ctx, const void* host_pinned_src, void* dev_dst, size_t bytes,
                          void* side_stream, void** event_out)
{
    DYMOE_REQUIRE(event_out != nullptr);
    *event_out = nullptr;
    if (bytes > 0) DYMOE_REQUIRE(host_pinned_src != nullptr && dev_dst != nullptr);
    if (!ctx) return DYMOE_ENOCTX;
    hipStream_t st = (hipStream_t)side_stream;
    hipEvent_t ev;
    if (hipEventCreateWithFlags(&ev, hipEventDisableTiming) != hipSuccess) return DYMOE_EHIP;
    if (bytes > 0 &&
        hipMemcpyAsync(dev_dst, host_pinned_src, bytes, hipMemcpyHostToDevice, st) != hipSuccess) {
        (void)hipEventDestroy(ev);
        return DYMOE_EHIP;
    }
    if (hipEventRecord(ev, st) != hipSuccess) {
        (void)hipEventDestroy(ev);
        return DYMOE_EHIP;
    }
    *event_out = (void*)ev;
    return DYMOE_OK;
}

int dymoe_prefetch_wait(dymoe_ctx* ctx, void* event, void* compute_stream)
{
    DYMOE_REQUIRE(event != nullptr);
    if (!ctx) return DYMOE_ENOCTX;
    if (hipStreamWaitEvent((hipStream_t)compute_stream, (hipEvent_t)event, 0) != hipSuccess) return DYMOE_EHIP;
    return DYMOE_OK;
}

int dymoe_prefetch_done(dymoe_ctx* ctx, void* event)
{
    DYMOE_REQUIRE(event != nullptr);
    if (!ctx) return DYMOE_ENOCTX;
    const hipError_t r = hipEventQuery((hipEvent_t)event);
    if (r == hipSuccess) return 1;
    if (r == hipErrorNotReady) return 0;
    return DYMOE_EHIP;
}

int dymoe_prefetch_release(dymoe_ctx* ctx, void* event)
{
    DYMOE_REQUIRE(event != nullptr);
    if (!ctx) return DYMOE_ENOCTX;
    return hipEventDestroy((hipEvent_t)event) == hipSuccess ? DYMOE_OK : DYMOE_EHIP;
}

int dymoe_residual_rmsnorm(dymoe_ctx* ctx, const void* h, const void* y, int y_dtype, float alpha,
                           int T, int H, void* h_out, void* stream)
{
    DYMOE_REQUIRE(T >= 0 && H > 0);
    DYMOE_REQUIRE(y_dtype == DYMOE_OUT_BF16 || y_dtype == DYMOE_OUT_F32);
    if (T > 0) DYMOE_REQUIRE(h && y && h_out);
    if (!ctx) return DYMOE_ENOCTX;
    if (T == 0) return DYMOE_OK;
    hipStream_t st = (hipStream_t)stream;
    const bool vec = H % 8 == 0 && dymoe_aligned(h, 16) && dymoe_aligned(y, 16) && dymoe_aligned(h_out, 16);
    const dim3 grid((unsigned)T), block(dymoe::kNormThreads);
#define DYMOE_NORM(YT_, VEC_)                                                                                         \
    hipLaunchKernelGGL((dymoe::residual_rmsnorm_kernel<YT_, VEC_>), grid, block, 0, st, (const uint16_t*)h,          \
                       (const YT_*)y, alpha, T, H, (uint16_t*)h_out)
    if (y_dtype == DYMOE_OUT_BF16) {
        if (vec) DYMOE_NORM(uint16_t, true);
        else DYMOE_NORM(uint16_t, false);
    } else {
        if (vec) DYMOE_NORM(float, true);
        else DYMOE_NORM(float, false);
    }
#undef DYMOE_NORM
    DYMOE_HIP_LAUNCH_CHECK();
    return DYMOE_OK;
}

}  // extern "C"
