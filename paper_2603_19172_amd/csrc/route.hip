// Router gating + top-k, and the activation-norm token score.
//
// route_kernel: a wavefront owns TW tokens; their activations stay in
// registers as packed bf16 pairs while the wavefront streams the router rows
// (16-byte loads, bf16 dot2 with fp32 accumulation).  Logits go to LDS, then
// the same wavefront does softmax and k rounds of arg-max (ties to the lower
// expert index) with cross-lane reductions.
#include <math.h>

#include "common.hpp"

namespace dymoe {

constexpr int kRouteWaves = 4;

template <int TW, int NCH>
__global__ __launch_bounds__(kRouteWaves* kWave) void route_kernel(
    const uint16_t* __restrict__ x, const uint16_t* __restrict__ wg,
    const float* __restrict__ bias, int T, int H, int E, int k, int renorm,
    int32_t* __restrict__ idx, float* __restrict__ w, float* __restrict__ probs)
{
    extern __shared__ float smem[];
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = threadIdx.x / kWave;
    float* logit = smem + (size_t)wave * TW * E;                 // [TW][E]
    float* selp = smem + (size_t)kRouteWaves * TW * E + (size_t)wave * k;  // [k]
    const int t0 = (blockIdx.x * kRouteWaves + wave) * TW;
    // wavefronts past the last token keep running on zero activations so that
    // every block-level barrier below is reached by all of them

    uint4 xr[TW][NCH];
#pragma unroll
    for (int tw = 0; tw < TW; tw++) {
#pragma unroll
        for (int c = 0; c < NCH; c++) {
            const int col = (c * kWave + lane) * 8;
            xr[tw][c] = make_uint4(0, 0, 0, 0);
            if (col < H && t0 + tw < T)
                xr[tw][c] = *reinterpret_cast<const uint4*>(x + (size_t)(t0 + tw) * H + col);
        }
    }
    for (int e = 0; e < E; e++) {
        float acc[TW];
#pragma unroll
        for (int tw = 0; tw < TW; tw++) acc[tw] = 0.0f;
        const uint16_t* row = wg + (size_t)e * H;
#pragma unroll
        for (int c = 0; c < NCH; c++) {
            const int col = (c * kWave + lane) * 8;
            if (c * kWave * 8 < H) {  // uniform
                uint4 wv = make_uint4(0, 0, 0, 0);
                if (col < H) wv = *reinterpret_cast<const uint4*>(row + col);
#pragma unroll
                for (int tw = 0; tw < TW; tw++) {
                    acc[tw] = dot2_bf16(wv.x, xr[tw][c].x, acc[tw]);
                    acc[tw] = dot2_bf16(wv.y, xr[tw][c].y, acc[tw]);
                    acc[tw] = dot2_bf16(wv.z, xr[tw][c].z, acc[tw]);
                    acc[tw] = dot2_bf16(wv.w, xr[tw][c].w, acc[tw]);
                }
            }
        }
        const float b = bias ? bias[e] : 0.0f;
#pragma unroll
        for (int tw = 0; tw < TW; tw++) {
            const float s = wave_sum(acc[tw]);
            if (lane == 0) logit[tw * E + e] = s + b;
        }
    }
    __syncthreads();

    for (int tw = 0; tw < TW; tw++) {
        const int t = t0 + tw;
        const bool valid = t < T;
        float* lg = logit + tw * E;
        float mx = -INFINITY;
        for (int e = lane; e < E; e += kWave) mx = fmaxf(mx, lg[e]);
        mx = wave_max(mx);
        float den = 0.0f;
        for (int e = lane; e < E; e += kWave) den += expf(lg[e] - mx);
        den = wave_sum(den);
        const float rden = 1.0f / den;
        if (probs && valid)
            for (int e = lane; e < E; e += kWave) probs[(size_t)t * E + e] = expf(lg[e] - mx) * rden;
        float sel_sum = 0.0f;
        for (int j = 0; j < k; j++) {
            float bv = -INFINITY;
            int bi = 0x7fffffff;
            for (int e = lane; e < E; e += kWave) {
                const float v = lg[e];
                if (v > bv || (v == bv && e < bi)) { bv = v; bi = e; }
            }
#pragma unroll
            for (int o = 32; o > 0; o >>= 1) {
                const float ov = __shfl_xor(bv, o, kWave);
                const int oi = __shfl_xor(bi, o, kWave);
                if (ov > bv || (ov == bv && oi < bi)) { bv = ov; bi = oi; }
            }
            // bi is now the same in every lane; the owner retires the entry
            const float p = expf(bv - mx) * rden;
            sel_sum += p;
            if (lane == 0) {
                if (valid) idx[(size_t)t * k + j] = bi;
                selp[j] = p;
            }
            if ((bi & (kWave - 1)) == lane) lg[bi] = -INFINITY;
            __syncthreads();
        }
        const float scale = renorm ? 1.0f / sel_sum : 1.0f;
        if (valid)
            for (int j = lane; j < k; j += kWave) w[(size_t)t * k + j] = selp[j] * scale;
        __syncthreads();
    }
}

// s_t = sqrt(sum_h x[t,h]^2), one wavefront per token
__global__ __launch_bounds__(256) void token_norm_kernel(const uint16_t* __restrict__ x, int T,
                                                         int H, float* __restrict__ score)
{
    const int lane = threadIdx.x & (kWave - 1);
    const int t = blockIdx.x * (256 / kWave) + threadIdx.x / kWave;
    if (t >= T) return;
    const uint16_t* row = x + (size_t)t * H;
    float acc = 0.0f;
    for (int col = lane * 8; col < H; col += kWave * 8) {
        const uint4 v = *reinterpret_cast<const uint4*>(row + col);
        const uint32_t u[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
        for (int i = 0; i < 4; i++) {
            const float a = bf16_lo(u[i]), b = bf16_hi(u[i]);
            acc = fmaf(a, a, acc);
            acc = fmaf(b, b, acc);
        }
    }
    acc = wave_sum(acc);
    if (lane == 0) score[t] = sqrtf(acc);
}

template <int TW, int NCH>
static int launch_route(dymoe_ctx* ctx, const void* x, const void* wg, const float* bias, int T, int H, int E,
                        int k, int renorm, int32_t* idx, float* w, float* probs, hipStream_t st)
{
    const int tokens_per_block = kRouteWaves * TW;
    const unsigned blocks = (unsigned)((T + tokens_per_block - 1) / tokens_per_block);
    const size_t smem = ((size_t)kRouteWaves * TW * E + (size_t)kRouteWaves * k) * sizeof(float);
    dymoe_kernel_timer timer(ctx, DYMOE_K_ROUTE, st);
    hipLaunchKernelGGL((route_kernel<TW, NCH>), dim3(blocks), dim3(kRouteWaves * kWave), smem, st,
                       (const uint16_t*)x, (const uint16_t*)wg, bias, T, H, E, k, renorm, idx, w,
                       probs);
    DYMOE_HIP_LAUNCH_CHECK();
    return DYMOE_OK;
}

}  // namespace dymoe

extern "C" {

int dymoe_route_topk(dymoe_ctx* ctx, const void* x, const void* wg, const float* bias,
                     int T, int H, int E, int k, int renorm,
                     int32_t* idx, float* w, float* probs, void* stream)
{
    DYMOE_REQUIRE(T >= 0 && H > 0 && E > 0 && k > 0 && k <= E);
    DYMOE_REQUIRE(H % 8 == 0);
    DYMOE_REQUIRE(wg != nullptr && dymoe_aligned(wg, 16));
    if (T > 0) DYMOE_REQUIRE(x && idx && w && dymoe_aligned(x, 16));  // empty step: nothing to read or write
    if (E > DYMOE_MAX_EXPERTS || H > 16384) return DYMOE_ENOTSUP;
    if (!ctx) return DYMOE_ENOCTX;
    if (T == 0) return DYMOE_OK;
    hipStream_t st = (hipStream_t)stream;
    // tokens per wavefront chosen so that their activations fit in 128 VGPRs;
    // few tokens: one per wavefront, to spread over more compute units
    if (H <= 4096 && T >= 1024 && E <= 256)
        return dymoe::launch_route<4, 8>(ctx, x, wg, bias, T, H, E, k, renorm, idx, w, probs, st);
    if (H <= 4096) return dymoe::launch_route<1, 8>(ctx, x, wg, bias, T, H, E, k, renorm, idx, w, probs, st);
    if (H <= 8192) return dymoe::launch_route<1, 16>(ctx, x, wg, bias, T, H, E, k, renorm, idx, w, probs, st);
    return dymoe::launch_route<1, 32>(ctx, x, wg, bias, T, H, E, k, renorm, idx, w, probs, st);
}

int dymoe_token_score_norm(dymoe_ctx* ctx, const void* x, int T, int H, float* score, void* stream)
{
    DYMOE_REQUIRE(T >= 0 && H > 0 && H % 8 == 0);
    if (T > 0) DYMOE_REQUIRE(x && score && dymoe_aligned(x, 16));
    if (!ctx) return DYMOE_ENOCTX;
    if (T == 0) return DYMOE_OK;
    const unsigned blocks = (unsigned)((T + 3) / 4);
    dymoe_kernel_timer timer(ctx, DYMOE_K_TOKEN_NORM, (hipStream_t)stream);
    hipLaunchKernelGGL(dymoe::token_norm_kernel, dim3(blocks), dim3(256), 0, (hipStream_t)stream,
                       (const uint16_t*)x, T, H, score);
    DYMOE_HIP_LAUNCH_CHECK();
    return DYMOE_OK;
}

}  // extern "C"
