// Router gating + top-k, and the activation-norm token score.
//
// route_kernel: a wavefront owns TW tokens; their activations stay in
// registers as packed bf16 pairs while the wavefront streams the router rows
// (16-byte loads, bf16 dot2 with fp32 accumulation).  Logits go to LDS, then
// the same wavefront does softmax and k rounds of arg-max (ties to the lower
// expert index) with cross-lane reductions.
#include <math.h>

#include "common.hpp"
#include "assign.hpp"

namespace dymoe {

// Logits of tokens t0 .. t0+TW-1 into LDS (logit[tw * E + e]).  Every wavefront
// of the workgroup keeps all TW activation rows in registers and computes the
// experts e = wave, wave + NW, ...
template <int TW, int NCH, int NW>
__device__ __forceinline__ void route_logits(const uint16_t* __restrict__ x,
                                             const uint16_t* __restrict__ wg,
                                             const float* __restrict__ bias, int T, int H, int E,
                                             int t0, float* logit)
{
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = threadIdx.x / kWave;
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
}

// Softmax and top-k of one token by one wavefront, from its logits in LDS (lg is
// consumed).  A wavefront only touches its own LDS rows here; LDS operations of
// one wavefront complete in order, so a wavefront-scope fence is all that the
// lane-to-lane hand-offs need.  prob_sum (LDS, may be null): prob_sum[e] += p[e];
// load_cnt (LDS, may be null): load_cnt[e] += 1 for the selected experts.
__device__ __forceinline__ void route_select(float* lg, float* selp, int t, int E, int k, int renorm,
                                             int32_t* __restrict__ idx, float* __restrict__ w,
                                             float* __restrict__ probs, float* prob_sum,
                                             int32_t* load_cnt)
{
    const int lane = threadIdx.x & (kWave - 1);
    float mx = -INFINITY;
    for (int e = lane; e < E; e += kWave) mx = fmaxf(mx, lg[e]);
    mx = wave_max(mx);
    float den = 0.0f;
    for (int e = lane; e < E; e += kWave) den += expf(lg[e] - mx);
    den = wave_sum(den);
    const float rden = 1.0f / den;
    if (probs || prob_sum)
        for (int e = lane; e < E; e += kWave) {
            const float p = expf(lg[e] - mx) * rden;
            if (probs) probs[(size_t)t * E + e] = p;
            if (prob_sum) prob_sum[e] += p;
        }
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
            if (load_cnt) load_cnt[bi] += 1;
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

// A workgroup of NW wavefronts owns TW tokens: logits by all wavefronts, then
// token tw is finished (softmax, top-k) by wavefront tw mod NW.  Few tokens:
// TW = 1 and the experts spread over 8 wavefronts; many tokens: TW = NW = 4, so
// that a router row is read once per four tokens.
template <int TW, int NCH, int NW>
__global__ __launch_bounds__(NW* kWave) void route_kernel(
    const uint16_t* __restrict__ x, const uint16_t* __restrict__ wg,
    const float* __restrict__ bias, int T, int H, int E, int k, int renorm,
    int32_t* __restrict__ idx, float* __restrict__ w, float* __restrict__ probs)
{
    extern __shared__ float smem[];
    const int wave = threadIdx.x / kWave;
    float* logit = smem;                                  // [TW][E]
    float* selp = smem + (size_t)TW * E + (size_t)wave * k;   // [NW][k]
    const int t0 = blockIdx.x * TW;
    route_logits<TW, NCH, NW>(x, wg, bias, T, H, E, t0, logit);
    __syncthreads();
    for (int tw = wave; tw < TW; tw += NW) {
        const int t = t0 + tw;
        if (t >= T) break;
        route_select(logit + tw * E, selp, t, E, k, renorm, idx, w, probs, nullptr, nullptr);
    }
}

// Decode step front end in one workgroup: for each of the (few) tokens the
// gating of route_kernel<1, NCH, 8>, then the decode importance (mean gate
// probability, summed in token order), the load histogram and the ranked
// bit-width assignment, with the arithmetic of the stand-alone kernels.
template <int NCH>
__global__ __launch_bounds__(8 * kWave) void decode_front_kernel(
    const uint16_t* __restrict__ x, const uint16_t* __restrict__ wg,
    const float* __restrict__ bias, int T, int H, int E, int k, int renorm,
    int32_t* __restrict__ idx, float* __restrict__ w, float* __restrict__ probs, TierTable tiers,
    int floor_bits, float* __restrict__ importance, int32_t* __restrict__ load,
    uint8_t* __restrict__ bits, int32_t* __restrict__ rank)
{
    extern __shared__ float smem[];
    __shared__ float s_imp[DYMOE_MAX_EXPERTS];
    __shared__ int32_t s_load[DYMOE_MAX_EXPERTS];
    const int wave = threadIdx.x / kWave;
    float* logit = smem;          // [E]
    float* selp = smem + E;       // [k]
    for (int e = threadIdx.x; e < E; e += blockDim.x) {
        s_imp[e] = 0.0f;
        s_load[e] = 0;
    }
    for (int t = 0; t < T; t++) {
        route_logits<1, NCH, 8>(x, wg, bias, T, H, E, t, logit);
        __syncthreads();
        if (wave == 0) route_select(logit, selp, t, E, k, renorm, idx, w, probs, s_imp, s_load);
        __syncthreads();
    }
    for (int e = threadIdx.x; e < E; e += blockDim.x) {
        const float g = s_imp[e];
        const float v = (T <= 1) ? g : g / (float)T;
        s_imp[e] = v;
        importance[e] = v;
        load[e] = s_load[e];
    }
    __syncthreads();
    for (int e = threadIdx.x; e < E; e += blockDim.x)
        assign_one<float>(e, E, s_imp, s_load, tiers, floor_bits, bits, rank);
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

int dymoe_decode_front(dymoe_ctx* ctx, const void* x, const void* wg, const float* bias,
                       int T, int H, int E, int k, int renorm, int n_tiers,
                       const int32_t* tier_count, const uint8_t* tier_bits, int floor_bits,
                       int32_t* idx, float* w, float* probs, float* importance, int32_t* load,
                       uint8_t* bits, int32_t* rank, void* stream)
{
    DYMOE_REQUIRE(T >= 1 && T <= DYMOE_FRONT_MAX_TOKENS && H > 0 && E > 0 && k > 0 && k <= E);
    DYMOE_REQUIRE(H % 8 == 0);
    DYMOE_REQUIRE(x && wg && idx && w && importance && load && bits);
    DYMOE_REQUIRE(dymoe_aligned(x, 16) && dymoe_aligned(wg, 16));
    DYMOE_REQUIRE(floor_bits == 0 || floor_bits == 2 || floor_bits == 4 || floor_bits == 8 || floor_bits == 16);
    dymoe::TierTable tt;
    DYMOE_REQUIRE(dymoe::make_tier_table(E, n_tiers, tier_count, tier_bits, tt) == DYMOE_OK);
    if (E > DYMOE_MAX_EXPERTS || H > 16384) return DYMOE_ENOTSUP;
    if (!ctx) return DYMOE_ENOCTX;
    hipStream_t st = (hipStream_t)stream;
    const size_t smem = ((size_t)E + (size_t)k) * sizeof(float);
    const uint16_t* xb = (const uint16_t*)x;
    const uint16_t* wb = (const uint16_t*)wg;
    if (H <= 4096)
        dymoe_launch(ctx, DYMOE_K_DECODE_FRONT, (dymoe::decode_front_kernel<8>), dim3(1), dim3(8 * dymoe::kWave), smem, st,
                     xb, wb, bias, T, H, E, k, renorm, idx, w, probs, tt, floor_bits, importance, load, bits, rank);
    else if (H <= 8192)
        dymoe_launch(ctx, DYMOE_K_DECODE_FRONT, (dymoe::decode_front_kernel<16>), dim3(1), dim3(8 * dymoe::kWave), smem, st,
                     xb, wb, bias, T, H, E, k, renorm, idx, w, probs, tt, floor_bits, importance, load, bits, rank);
    else
        dymoe_launch(ctx, DYMOE_K_DECODE_FRONT, (dymoe::decode_front_kernel<32>), dim3(1), dim3(8 * dymoe::kWave), smem, st,
                     xb, wb, bias, T, H, E, k, renorm, idx, w, probs, tt, floor_bits, importance, load, bits, rank);
    DYMOE_HIP_LAUNCH_CHECK();
    return DYMOE_OK;
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
