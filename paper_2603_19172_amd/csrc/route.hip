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

// A workgroup of NW wavefronts owns TW tokens.  Every wavefront keeps all TW
// activation rows in registers and computes the logits of the experts
// e = wave, wave + NW, ...; then token tw is finished (softmax, top-k) by
// wavefront tw mod NW.  Few tokens: TW = 1 and the experts spread over 8
// wavefronts; many tokens: TW = NW = 4, so that a router row is read once per
// four tokens.
template <int TW, int NCH, int NW>
__global__ __launch_bounds__(NW* kWave) void route_kernel(
    const uint16_t* __restrict__ x, const uint16_t* __restrict__ wg,
    const float* __restrict__ bias, int T, int H, int E, int k, int renorm,
    int32_t* __restrict__ idx, float* __restrict__ w, float* __restrict__ probs)
{
    extern __shared__ float smem[];
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = threadIdx.x / kWave;
    float* logit = smem;                                  // [TW][E]
    float* selp = smem + (size_t)TW * E + (size_t)wave * k;   // [NW][k]
    const int t0 = blockIdx.x * TW;

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
    for (int e = wave; e < E; e += NW) {
        float acc[TW];
#pragma unroll
        for (int tw = 0; tw < TW; tw++) acc[tw] = 0.0f;
        const uint16_t* row = wg + (size_t)e * H;
#pragma unroll
        for (int c = 0; c < NCH; c++) {
            if (c * kWave * 8 < H) {  // uniform
                // lanes past the end re-read the row's tail against zero activations
                const int col = min((c * kWave + lane) * 8, H - 8);
                const uint4 wv = *reinterpret_cast<const uint4*>(row + col);
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

    // From here on a wavefront only touches the LDS rows of its own tokens; LDS
    // operations of one wavefront complete in order, so a wavefront-scope fence
    // is all that the lane-to-lane hand-offs below need.
    for (int tw = wave; tw < TW; tw += NW) {
        const int t = t0 + tw;
        if (t >= T) break;
        float* lg = logit + tw * E;
        float mx = -INFINITY;
        for (int e = lane; e < E; e += kWave) mx = fmaxf(mx, lg[e]);
        mx = wave_max(mx);
        float den = 0.0f;
        for (int e = lane; e < E; e += kWave) den += expf(lg[e] - mx);
        den = wave_sum(den);
        const float rden = 1.0f / den;
        if (probs)
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
                idx[(size_t)t * k + j] = bi;
                selp[j] = p;
            }
            if ((bi & (kWave - 1)) == lane) lg[bi] = -INFINITY;
            __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "wavefront");
            __builtin_amdgcn_wave_barrier();
        }
        const float scale = renorm ? 1.0f / sel_sum : 1.0f;
        for (int j = lane; j < k; j += kWave) w[(size_t)t * k + j] = selp[j] * scale;
        __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "wavefront");
        __builtin_amdgcn_wave_barrier();
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

template <int TW, int NCH, int NW>
static int launch_route(dymoe_ctx* ctx, const void* x, const void* wg, const float* bias, int T, int H, int E,
                        int k, int renorm, int32_t* idx, float* w, float* probs, hipStream_t st)
{
    const unsigned blocks = (unsigned)((T + TW - 1) / TW);
    const size_t smem = ((size_t)TW * E + (size_t)NW * k) * sizeof(float);
    dymoe_launch(ctx, DYMOE_K_ROUTE, (route_kernel<TW, NCH, NW>), dim3(blocks), dim3(NW * kWave), smem, st,
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
    // tokens per workgroup chosen so that their activations fit in 128 VGPRs;
    // few tokens: one per workgroup, its experts spread over 8 wavefronts
    if (H <= 4096 && T >= 1024)
        return dymoe::launch_route<4, 8, 4>(ctx, x, wg, bias, T, H, E, k, renorm, idx, w, probs, st);
    if (H <= 4096) return dymoe::launch_route<1, 8, 8>(ctx, x, wg, bias, T, H, E, k, renorm, idx, w, probs, st);
    if (H <= 8192) return dymoe::launch_route<1, 16, 8>(ctx, x, wg, bias, T, H, E, k, renorm, idx, w, probs, st);
    return dymoe::launch_route<1, 32, 8>(ctx, x, wg, bias, T, H, E, k, renorm, idx, w, probs, st);
}

int dymoe_token_score_norm(dymoe_ctx* ctx, const void* x, int T, int H, float* score, void* stream)
{
    DYMOE_REQUIRE(T >= 0 && H > 0 && H % 8 == 0);
    if (T > 0) DYMOE_REQUIRE(x && score && dymoe_aligned(x, 16));
    if (!ctx) return DYMOE_ENOCTX;
    if (T == 0) return DYMOE_OK;
    const unsigned blocks = (unsigned)((T + 3) / 4);
    dymoe_launch(ctx, DYMOE_K_TOKEN_NORM, dymoe::token_norm_kernel, dim3(blocks), dim3(256), 0, (hipStream_t)stream,
                       (const uint16_t*)x, T, H, score);
    DYMOE_HIP_LAUNCH_CHECK();
    return DYMOE_OK;
}

}  // extern "C"
