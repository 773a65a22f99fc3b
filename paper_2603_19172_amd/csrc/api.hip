// Context, error text, workspace size and the host-side depth schedule.
#include <math.h>
#include <new>

#include "common.hpp"
#include "ffn_layout.hpp"

namespace dymoe {

// Plain copy, 16 bytes per lane, every wavefront instruction moving 1 KiB of
// contiguous memory: the access pattern of the weight-streaming kernels, with
// exactly known traffic.
__global__ __launch_bounds__(256) void stream_copy_kernel(const uint4* __restrict__ src,
                                                          uint4* __restrict__ dst, long n16)
{
    const long i = (long)blockIdx.x * 1024 + threadIdx.x;
    uint4 v[4];
#pragma unroll
    for (int u = 0; u < 4; u++)
        if (i + 256 * u < n16) v[u] = src[i + 256 * u];
#pragma unroll
    for (int u = 0; u < 4; u++)
        if (i + 256 * u < n16) dst[i + 256 * u] = v[u];
}

// Register-only loop of bf16 matrix instructions: every wavefront keeps four independent accumulators busy with
// v_mfma_f32_32x32x16_bf16 and touches no memory until the end.  What it sustains is the matrix rate this chip
// reaches at the clock it holds under that load, the practical ceiling beside the data sheet's figure.
__global__ __launch_bounds__(256) void mfma_peak_kernel(float* __restrict__ sink, int iters)
{
    typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
    typedef float f32x16 __attribute__((ext_vector_type(16)));
    const int tid = blockIdx.x * 256 + threadIdx.x;
    bf16x8 a, b;
#pragma unroll
    for (int i = 0; i < 8; i++) {
        a[i] = (__bf16)(float)((tid + i) & 7) * (__bf16)0.125f;
        b[i] = (__bf16)(float)((tid + 3 * i) & 3) * (__bf16)0.25f;
    }
    f32x16 c0 = {0}, c1 = {0}, c2 = {0}, c3 = {0};
    for (int it = 0; it < iters; it++) {
        c0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c0, 0, 0, 0);
        c1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c1, 0, 0, 0);
        c2 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c2, 0, 0, 0);
        c3 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c3, 0, 0, 0);
    }
    sink[tid] = c0[0] + c1[5] + c2[10] + c3[15];
}

int ffn_static_scratch_address(void** out);
int ffn_device_flags_address(unsigned** out);
int ffn_gemm_init();
int route_init();

}  // namespace dymoe

extern "C" {

int dymoe_stream_copy(dymoe_ctx* ctx, const void* src, void* dst, size_t bytes, void* stream)
{
    DYMOE_REQUIRE(bytes % 16 == 0);
    if (bytes == 0) return DYMOE_OK;
    DYMOE_REQUIRE(src != nullptr && dst != nullptr && dymoe_aligned(src, 16) && dymoe_aligned(dst, 16));
    if (!ctx) return DYMOE_ENOCTX;
    const long n16 = (long)(bytes / 16);
    const long blocks = (n16 + 1023) / 1024;
    DYMOE_REQUIRE(blocks <= 0x7fffffffL);
    dymoe_launch(ctx, DYMOE_K_STREAM_COPY, dymoe::stream_copy_kernel, dim3((unsigned)blocks), dim3(256), 0,
                 (hipStream_t)stream, (const uint4*)src, (uint4*)dst, n16);
    DYMOE_HIP_LAUNCH_CHECK();
    return DYMOE_OK;
}

int dymoe_mfma_peak(dymoe_ctx* ctx, int iters, int waves_per_simd, float* sink, size_t sink_floats, double* flops,
                    void* stream)
{
    DYMOE_REQUIRE(iters > 0 && (waves_per_simd == 1 || waves_per_simd == 2) && sink != nullptr);
    if (!ctx) return DYMOE_ENOCTX;
    const unsigned blocks = (unsigned)(ctx->num_cu * waves_per_simd);     // four wavefronts each, one per SIMD
    DYMOE_REQUIRE(sink_floats >= (size_t)blocks * 256);
    dymoe_launch(ctx, DYMOE_K_MFMA_PEAK, dymoe::mfma_peak_kernel, dim3(blocks), dim3(256), 0, (hipStream_t)stream, sink,
                 iters);
    DYMOE_HIP_LAUNCH_CHECK();
    if (flops) *flops = (double)blocks * 4.0 * (double)iters * 4.0 * (2.0 * 32 * 32 * 16);
    return DYMOE_OK;
}

int dymoe_create(dymoe_ctx** out, int device)
{
    DYMOE_REQUIRE(out != nullptr && device >= 0);
    *out = nullptr;
    int n = 0;
    if (hipGetDeviceCount(&n) != hipSuccess || device >= n) return DYMOE_EHIP;
    hipDeviceProp_t prop;
    if (hipGetDeviceProperties(&prop, device) != hipSuccess) return DYMOE_EHIP;
    dymoe_ctx* c = new (std::nothrow) dymoe_ctx;
    if (!c) return DYMOE_EHIP;
    c->device = device;
    c->num_cu = prop.multiProcessorCount;
    c->timing_mask = 0;
    c->static_scratch = nullptr;
    c->device_flags = nullptr;
    // per-device set-up, with that device current: the address of its copy of the static scratch array, and the
    // dynamic-LDS limits of the grouped-GEMM and matrix-core router kernels (so that no later call has anything left to configure)
    int prev = 0;
    int rc = DYMOE_OK;
    if (hipGetDevice(&prev) != hipSuccess || hipSetDevice(device) != hipSuccess) rc = DYMOE_EHIP;
    if (rc == DYMOE_OK) {
        rc = dymoe::ffn_static_scratch_address(&c->static_scratch);
        if (rc == DYMOE_OK) rc = dymoe::ffn_device_flags_address(&c->device_flags);
        if (rc == DYMOE_OK) rc = dymoe::ffn_gemm_init();
        if (rc == DYMOE_OK) rc = dymoe::route_init();
        if (hipSetDevice(prev) != hipSuccess) rc = DYMOE_EHIP;
    }
    if (rc != DYMOE_OK) {
        delete c;
        return rc;
    }
    *out = c;
    return DYMOE_OK;
}

int dymoe_device_flags(dymoe_ctx* ctx, unsigned* flags, void* stream)
{
    DYMOE_REQUIRE(flags != nullptr);
    if (!ctx) return DYMOE_ENOCTX;
    if (!ctx->device_flags) return DYMOE_EHIP;
    hipStream_t st = (hipStream_t)stream;
    unsigned v = 0;
    if (hipMemcpyAsync(&v, ctx->device_flags, sizeof(v), hipMemcpyDeviceToHost, st) != hipSuccess) return DYMOE_EHIP;
    if (hipStreamSynchronize(st) != hipSuccess) return DYMOE_EHIP;
    if (v != 0) {
        if (hipMemsetAsync(ctx->device_flags, 0, sizeof(v), st) != hipSuccess) return DYMOE_EHIP;
        if (hipStreamSynchronize(st) != hipSuccess) return DYMOE_EHIP;
    }
    *flags = v;
    return DYMOE_OK;
}

int dymoe_format_present(const dymoe_expert_fmt* entry, int bits)
{
    if (!entry) return 0;
    return dymoe_fmt_present(*entry, bits) ? 1 : 0;
}

static void drop_timed(dymoe_ctx* ctx)
{
    for (auto& t : ctx->timed) {
        (void)hipEventDestroy(t.start);
        (void)hipEventDestroy(t.stop);
    }
    ctx->timed.clear();
}

void dymoe_destroy(dymoe_ctx* ctx)
{
    if (!ctx) return;
    drop_timed(ctx);
    delete ctx;
}

int dymoe_timing_enable(dymoe_ctx* ctx, unsigned kernel_mask)
{
    if (!ctx) return DYMOE_ENOCTX;
    DYMOE_REQUIRE((kernel_mask >> DYMOE_K_COUNT) == 0);
    drop_timed(ctx);
    ctx->timing_mask = kernel_mask;
    return DYMOE_OK;
}

int dymoe_timing_read(dymoe_ctx* ctx, int kernel, double* total_ms, int* launches)
{
    DYMOE_REQUIRE(kernel >= 0 && kernel < DYMOE_K_COUNT && total_ms && launches);
    if (!ctx) return DYMOE_ENOCTX;
    double sum = 0.0;
    int n = 0;
    std::vector<dymoe_timed_launch> rest;
    int rc = DYMOE_OK;
    for (auto& t : ctx->timed) {
        if (t.kernel != kernel) {
            rest.push_back(t);
            continue;
        }
        float ms = 0.0f;
        if (hipEventSynchronize(t.stop) != hipSuccess || hipEventElapsedTime(&ms, t.start, t.stop) != hipSuccess)
            rc = DYMOE_EHIP;
        sum += (double)ms;
        n++;
        (void)hipEventDestroy(t.start);      // a record is read once
        (void)hipEventDestroy(t.stop);
    }
    ctx->timed.swap(rest);
    *total_ms = sum;
    *launches = n;
    return rc;
}

const char* dymoe_kernel_name(int kernel)
{
    switch (kernel) {
    case DYMOE_K_ROUTE: return "route_kernel";
    case DYMOE_K_TOKEN_NORM: return "token_norm_kernel";
    case DYMOE_K_IMPORTANCE: return "importance_prefill_kernel";
    case DYMOE_K_ASSIGN: return "assign_precision_kernel";
    case DYMOE_K_QUANTIZE: return "quantize_experts_kernel";
    case DYMOE_K_GEMV_PHASE1: return "gemv_phase1_kernel";
    case DYMOE_K_GEMV_PHASE2: return "gemv_phase2_kernel";
    case DYMOE_K_GEMV_COMBINE: return "gemv_combine_kernel";
    case DYMOE_K_PLAN: return "plan_kernel";
    case DYMOE_K_GEMM1: return "gemm_kernel<1>";
    case DYMOE_K_GEMM2: return "gemm_kernel<2>";
    case DYMOE_K_GEMM_COMBINE: return "gemm_combine_kernel";
    case DYMOE_K_STREAM_COPY: return "stream_copy_kernel";
    case DYMOE_K_DECODE_FRONT: return "decode_front_kernel";
    case DYMOE_K_ATTN_STATS: return "attn_rowstats_kernel";
    case DYMOE_K_ATTN_COLSUM: return "attn_colsum_kernel";
    case DYMOE_K_GPTQ_GROUP: return "gptq_group_kernel";
    case DYMOE_K_GPTQ_TRAIL: return "gptq_trail_kernel";
    case DYMOE_K_GPTQ_HESSIAN: return "gptq_hessian_kernel";
    case DYMOE_K_GPTQ_FACTOR: return "gptq_chol_diag_kernel";
    case DYMOE_K_MFMA_PEAK: return "mfma_peak_kernel";
    case DYMOE_K_ROUTE_SELECT: return "route_select_kernel";
    default: return nullptr;
    }
}

const char* dymoe_strerror(int code)
{
    switch (code) {
    case DYMOE_OK: return "success";
    case DYMOE_EINVAL: return "invalid argument";
    case DYMOE_ENOSPC: return "workspace too small";
    case DYMOE_EHIP: return "HIP runtime call failed";
    case DYMOE_ENOTSUP: return "size or mode not supported by the kernels";
    case DYMOE_ENOCTX: return "context is NULL";
    default: return "unknown error code";
    }
}

size_t dymoe_workspace_bytes(int T, int H, int F, int E, int k)
{
    if (T < 0 || H <= 0 || F <= 0 || E <= 0 || k <= 0 || k > E) return 0;
    return dymoe::ffn_layout(T, H, F, E, k).total;
}

size_t dymoe_ffn_plan_offset(int T, int H, int F, int E, int k)
{
    if (T < 0 || H <= 0 || F <= 0 || E <= 0 || k <= 0 || k > E) return 0;
    return dymoe::ffn_layout(T, H, F, E, k).plan;
}

// Paper Sec. 4.3: cosine retention ratio, then the ceiling.  The product is
// lowered by 1e-9 before the ceiling so that an exactly integral r(l)*M that
// evaluates one ulp high (cos(pi/3) = 0.5000000000000001) is not rounded up.
int dymoe_depth_schedule(int layer, int n_layers, double lambda, int M)
{
    if (M < 1 || n_layers < 1 || layer < 0 || layer >= n_layers) return DYMOE_EINVAL;
    if (!(lambda >= 0.0 && lambda <= 1.0)) return DYMOE_EINVAL;
    double r = 1.0;
    if (n_layers > 1) {
        const double kPi = 3.141592653589793238462643383279502884;
        double c = cos(kPi * (double)layer / (double)(n_layers - 1));
        r = (1.0 - lambda) * 0.5 * (c + 1.0) + lambda;
    }
    double t = ceil(r * (double)M - 1e-9);
    if (t < 1.0) t = 1.0;
    if (t > (double)M) t = (double)M;
    return (int)t;
}

}  // extern "C"
