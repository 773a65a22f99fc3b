// Host-resident experts: copies from pinned host memory into device buffers on
// a side stream, handed over to the compute stream through events, and the
// residual + normalisation step that chains layers of a stack.
#include <math.h>

#include "common.hpp"

namespace dymoe {

// v = h[t,:] + alpha * y[t,:];  h_out[t,:] = bf16(v / rms(v)), one wavefront per token, fp32 arithmetic
template <typename YT>
__global__ __launch_bounds__(256) void residual_rmsnorm_kernel(const uint16_t* __restrict__ h,
                                                              const YT* __restrict__ y, float alpha,
                                                              int T, int H, uint16_t* __restrict__ out)
{
    const int lane = threadIdx.x & (kWave - 1);
    const int t = blockIdx.x * (256 / kWave) + threadIdx.x / kWave;
    if (t >= T) return;
    const uint16_t* hr = h + (size_t)t * H;
    const YT* yr = y + (size_t)t * H;
    float ss = 0.0f;
    for (int j = lane; j < H; j += kWave) {
        float yv;
        if constexpr (sizeof(YT) == 2) yv = bf16_bits_to_f32(yr[j]);
        else yv = yr[j];
        const float v = fmaf(alpha, yv, bf16_bits_to_f32(hr[j]));
        ss = fmaf(v, v, ss);
    }
    ss = wave_sum(ss);
    const float inv = (ss > 0.0f) ? 1.0f / sqrtf(ss / (float)H) : 0.0f;
    uint16_t* orow = out + (size_t)t * H;
    for (int j = lane; j < H; j += kWave) {
        float yv;
        if constexpr (sizeof(YT) == 2) yv = bf16_bits_to_f32(yr[j]);
        else yv = yr[j];
        const float v = fmaf(alpha, yv, bf16_bits_to_f32(hr[j]));
        orow[j] = (uint16_t)f32_to_bf16_bits(v * inv);
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
    const unsigned blocks = (unsigned)((T + 3) / 4);
    hipStream_t st = (hipStream_t)stream;
    if (y_dtype == DYMOE_OUT_BF16)
        hipLaunchKernelGGL(dymoe::residual_rmsnorm_kernel<uint16_t>, dim3(blocks), dim3(256), 0, st,
                           (const uint16_t*)h, (const uint16_t*)y, alpha, T, H, (uint16_t*)h_out);
    else
        hipLaunchKernelGGL(dymoe::residual_rmsnorm_kernel<float>, dim3(blocks), dim3(256), 0, st,
                           (const uint16_t*)h, (const float*)y, alpha, T, H, (uint16_t*)h_out);
    DYMOE_HIP_LAUNCH_CHECK();
    return DYMOE_OK;
}

}  // extern "C"
