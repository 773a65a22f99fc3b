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
#include "route_device.hpp"

namespace dymoe {

// the same with NC chosen for E (E <= DYMOE_MAX_EXPERTS = 1024)
template <int TB>
__device__ __forceinline__ void route_select_batch(float* const (&lg)[TB], float* const (&selp)[TB],
                                                   const int (&t)[TB], int E, int k, int renorm,
                                                   int32_t* __restrict__ idx, float* __restrict__ w,
                                                   float* probs, float* prob_sum,
                                                   int32_t* load_cnt)
{
    if (E <= 64) route_select_regs<TB, 1>(lg, selp, t, E, k, renorm, idx, w, probs, prob_sum, load_cnt);
    else if (E <= 128) route_select_regs<TB, 2>(lg, selp, t, E, k, renorm, idx, w, probs, prob_sum, load_cnt);
    else if (E <= 256) route_select_regs<TB, 4>(lg, selp, t, E, k, renorm, idx, w, probs, prob_sum, load_cnt);
    else if (E <= 512) route_select_regs<TB, 8>(lg, selp, t, E, k, renorm, idx, w, probs, prob_sum, load_cnt);
    else route_select_regs<TB, 16>(lg, selp, t, E, k, renorm, idx, w, probs, prob_sum, load_cnt);
}

// one token
__device__ __forceinline__ void route_select(float* lg, float* selp, int t, int E, int k, int renorm,
                                             int32_t* __restrict__ idx, float* __restrict__ w,
                                             float* probs, float* prob_sum,
                                             int32_t* load_cnt)
{
    float* const lgs[1] = {lg};
    float* const sps[1] = {selp};
    const int ts[1] = {t};
    route_select_batch<1>(lgs, sps, ts, E, k, renorm, idx, w, probs, prob_sum, load_cnt);
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

// Gating of many tokens against many experts: the logits are a dense contraction
// [T,H] x [H,E], done on the matrix cores.  A workgroup of eight wavefronts owns 32
// tokens and takes the experts 128 at a time (four 32-expert fragments).  Both
// operands are rows of length H in memory, and an MFMA operand wants a lane per row:
// read that way every load instruction touches 32 or 64 different cache lines for a
// few bytes of each, and the texture path, which works a line at a time, becomes the
// limit (measured: 33 of the kernel's 50 us).  So the operands go through LDS: per
// K-tile of 128 columns the workgroup reads 32 token rows and 128 router rows with
// 16 lanes per row (a wavefront instruction covers 4 rows x 256 contiguous bytes),
// one K-tile ahead into registers, and stores them with the 16-byte chunk c of row r
// at chunk position c ^ (r & 15), so that the operand reads (a lane per row, fixed c)
// fall on all banks once.  Wavefront w multiplies expert fragment w % 4 over half
// w / 4 of each K-tile's eight 16-column steps; the two halves meet in LDS and are
// added in that order.  Tiles are computed transposed (experts down, tokens across):
// a lane then holds one token's logits of 16 experts.  Softmax and top-k are
// route_select's, four tokens side by side per wavefront.
constexpr int kRmTokens = 32;
constexpr int kRmExperts = 128;
constexpr int kRmWaves = 8;
constexpr int kRmThreads = kRmWaves * kWave;
constexpr int kRmBK = 128;       // columns per K-tile
constexpr int kRmBatch = 4;      // tokens a wavefront takes through softmax and top-k side by side
constexpr int kRmWChunks = kRmExperts * (kRmBK / 8) / kRmThreads;      // 16-byte chunks of router rows per thread and K-tile

__global__ __launch_bounds__(kRmThreads) void route_mfma_kernel(
    const uint16_t* __restrict__ x, const uint16_t* __restrict__ wg,
    const float* __restrict__ bias, int T, int H, int E, int k, int renorm,
    int32_t* __restrict__ idx, float* __restrict__ w, float* __restrict__ probs)
{
    extern __shared__ __attribute__((aligned(1024))) float smem[];
    static_assert(kRmTokens * (kRmBK / 8) == kRmThreads, "one chunk of the token tile per thread");
    const int tid = threadIdx.x;
    const int lane = tid & (kWave - 1), wave = tid / kWave;
    const int ln = lane & 31, kb = lane >> 5;
    char* xs = reinterpret_cast<char*>(smem);                       // [32 rows][256 bytes], swizzled
    char* ws = xs + kRmTokens * kRmBK * 2;                          // [128 rows][256 bytes], swizzled
    float* part = reinterpret_cast<float*>(ws + kRmExperts * kRmBK * 2);   // [2 halves][32 tokens][128 experts]
    float* logit = part + 2 * kRmTokens * kRmExperts;               // [32 tokens][E]
    float* selp = logit + (size_t)kRmTokens * E + (size_t)wave * kRmBatch * k;   // [8 wavefronts][kRmBatch][k]
    const int t0 = blockIdx.x * kRmTokens;
    const int n_kt = H / kRmBK;
    // staging role: chunk (tid % 16) of row (tid / 16) of the token tile, and of router rows tid / 16 + 32 u
    const int s_row = tid >> 4, s_chunk = tid & 15;
    const uint16_t* x_src = x + (size_t)min(t0 + s_row, T - 1) * H + s_chunk * 8;
    const uint32_t s_off = (uint32_t)(s_row * (kRmBK * 2) + ((s_chunk ^ (s_row & 15)) << 4));   // the same swizzle for rows 32 u apart
    // operand role: fragment f, K half h; lane (ln, kb) reads row ln (token) or 32 f + ln (expert), chunk 2 j + kb
    const int f = wave & 3, h = wave >> 2;
    const uint32_t a_off = (uint32_t)((32 * f + ln) * (kRmBK * 2));
    const uint32_t b_off = (uint32_t)(ln * (kRmBK * 2));
    const uint32_t sw = (uint32_t)(ln & 15);
    for (int e0 = 0; e0 < E; e0 += kRmExperts) {
        const uint16_t* w_src[kRmWChunks];
#pragma unroll
        for (int u = 0; u < kRmWChunks; u++) w_src[u] = wg + (size_t)min(e0 + s_row + 32 * u, E - 1) * H + s_chunk * 8;
        float16_t acc;
#pragma unroll
        for (int i = 0; i < 16; i++) acc[i] = 0.0f;
        uint4 xr, wr[kRmWChunks];
        xr = load_global<uint4>(x_src);
#pragma unroll
        for (int u = 0; u < kRmWChunks; u++) wr[u] = load_global<uint4>(w_src[u]);
        for (int kt = 0; kt < n_kt; kt++) {
            __syncthreads();                    // the previous tile has been read by every wavefront
            *reinterpret_cast<uint4*>(xs + s_off) = xr;
#pragma unroll
            for (int u = 0; u < kRmWChunks; u++) *reinterpret_cast<uint4*>(ws + s_off + u * (32 * kRmBK * 2)) = wr[u];
            // the next K-tile's rows, in flight while this one is multiplied (past the end: the last one again, unused)
            const int kn = min(kt + 1, n_kt - 1);
            xr = load_global<uint4>(x_src + kn * kRmBK);
#pragma unroll
            for (int u = 0; u < kRmWChunks; u++) wr[u] = load_global<uint4>(w_src[u] + kn * kRmBK);
            __syncthreads();
#pragma unroll
            for (int j = 4 * h; j < 4 * h + 4; j++) {
                const uint32_t c = ((uint32_t)(2 * j + kb) ^ sw) << 4;
                const uint4 av = *reinterpret_cast<const uint4*>(ws + a_off + c);
                const uint4 bv = *reinterpret_cast<const uint4*>(xs + b_off + c);
                acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, av), __builtin_bit_cast(bf16x8_t, bv),
                                                             acc, 0, 0, 0);
            }
        }
        // register i: expert 32 f + 8 (i / 4) + 4 kb + i % 4, token ln
        float* mine = part + ((size_t)h * kRmTokens + ln) * kRmExperts + 32 * f;
#pragma unroll
        for (int g = 0; g < 4; g++)
            *reinterpret_cast<float4*>(mine + 8 * g + 4 * kb) = make_float4(acc[4 * g], acc[4 * g + 1], acc[4 * g + 2], acc[4 * g + 3]);
        __syncthreads();
        for (int i = tid; i < kRmTokens * kRmExperts; i += kRmThreads) {
            const int tok = i / kRmExperts, e = e0 + i % kRmExperts;
            if (e < E) logit[(size_t)tok * E + e] = (part[i] + part[kRmTokens * kRmExperts + i]) + (bias ? bias[e] : 0.0f);
        }
        __syncthreads();
    }
    // wavefront `wave` finishes tokens wave, wave + 8, wave + 16, wave + 24, side by side
    {
        float* lgs[kRmBatch];
        float* sps[kRmBatch];
        int ts[kRmBatch];
#pragma unroll
        for (int b = 0; b < kRmBatch; b++) {
            const int tw = wave + kRmWaves * b;
            lgs[b] = logit + (size_t)tw * E;
            sps[b] = selp + b * k;
            ts[b] = (t0 + tw < T) ? t0 + tw : -1;      // rows past the last token hold a copy of it: computed, not stored
        }
        float* const (&lgc)[kRmBatch] = lgs;
        float* const (&spc)[kRmBatch] = sps;
        route_select_batch<kRmBatch>(lgc, spc, ts, E, k, renorm, idx, w, probs, nullptr, nullptr);
    }
}

// The same gating when the token tiles are fewer than the compute units (2048 tokens make 64): cut by experts
// as well.  route_logits_kernel: a workgroup of four wavefronts takes 32 tokens x 32 experts (a quarter of the
// router rows per workgroup instead of all of them: the rows a workgroup has to pull in, not the arithmetic, are what
// the one-kernel form spends its time on), each wavefront a quarter of every K-tile's 16-column steps; the four
// partial tiles meet in LDS, in the operand tile's place, and are added in wavefront order; logits (+ bias) go to
// memory.  route_select_kernel: softmax and top-k of 32 tokens per workgroup from those logits, as above.
constexpr int kRlWaves = 4;
constexpr int kRlThreads = kRlWaves * kWave;
#ifndef DYMOE_RL_BK
#define DYMOE_RL_BK 256
#endif
constexpr int kRlBK = DYMOE_RL_BK;       // columns per K-tile

template <int BK>
__global__ __launch_bounds__(kRlThreads) void route_logits_kernel(
    const uint16_t* __restrict__ x, const uint16_t* __restrict__ wg, const float* __restrict__ bias,
    int T, int H, int E, float* __restrict__ logit)
{
    // rows 0..31: tokens, 32..63: router rows; 2 BK bytes each, 16-byte chunk c of row r at chunk position c ^ (r & 15)
    constexpr int kRowBytes = 2 * BK, kRowChunks = BK / 8;
    constexpr int kRowsPerPass = kRlThreads / kRowChunks, kPasses = 64 / kRowsPerPass;
    __shared__ __attribute__((aligned(1024))) char tiles[64 * kRowBytes];
    static_assert(sizeof(tiles) >= kRlWaves * 32 * 32 * sizeof(float), "the partial tiles fit in the operand tile");
    const int tid = threadIdx.x;
    const int lane = tid & (kWave - 1), wave = tid / kWave;
    const int ln = lane & 31, kb = lane >> 5;
    const int t0 = blockIdx.x * 32, e0 = blockIdx.y * 32;
    const int n_kt = H / BK;
    // staging role: chunk tid % kRowChunks of rows tid / kRowChunks + kRowsPerPass u
    const int s_row = tid / kRowChunks, s_chunk = tid % kRowChunks;
    const uint16_t* src[kPasses];
    uint32_t s_off[kPasses];
#pragma unroll
    for (int u = 0; u < kPasses; u++) {
        const int row = s_row + kRowsPerPass * u;
        src[u] = ((row < 32) ? x + (size_t)min(t0 + row, T - 1) * H : wg + (size_t)min(e0 + row - 32, E - 1) * H) + s_chunk * 8;
        s_off[u] = (uint32_t)(row * kRowBytes + ((s_chunk ^ (row & 15)) << 4));
    }
    const uint32_t a_off = (uint32_t)((32 + ln) * kRowBytes);
    const uint32_t b_off = (uint32_t)(ln * kRowBytes);
    const uint32_t sw = (uint32_t)(ln & 15);
    constexpr int kSteps = BK / 16 / kRlWaves;      // 16-column MFMA steps per wavefront and K-tile
    float16_t acc;
#pragma unroll
    for (int i = 0; i < 16; i++) acc[i] = 0.0f;
    uint4 r[kPasses];
#pragma unroll
    for (int u = 0; u < kPasses; u++) r[u] = load_global<uint4>(src[u]);
    for (int kt = 0; kt < n_kt; kt++) {
        __syncthreads();                    // the previous tile has been read by every wavefront
#pragma unroll
        for (int u = 0; u < kPasses; u++) *reinterpret_cast<uint4*>(tiles + s_off[u]) = r[u];
        // the next K-tile's rows, in flight while this one is multiplied (past the end: the last one again, unused)
        const int kn = min(kt + 1, n_kt - 1);
#pragma unroll
        for (int u = 0; u < kPasses; u++) r[u] = load_global<uint4>(src[u] + kn * BK);
        __syncthreads();
#pragma unroll
        for (int j = kSteps * wave; j < kSteps * wave + kSteps; j++) {
            const uint32_t c = ((uint32_t)(2 * j + kb) ^ sw) << 4;
            const uint4 av = *reinterpret_cast<const uint4*>(tiles + a_off + c);
            const uint4 bv = *reinterpret_cast<const uint4*>(tiles + b_off + c);
            acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, av), __builtin_bit_cast(bf16x8_t, bv),
                                                         acc, 0, 0, 0);
        }
    }
    __syncthreads();                        // the last tile has been read: its place takes the partial tiles
    // register i: expert 8 (i / 4) + 4 kb + i % 4, token ln
    float* part = reinterpret_cast<float*>(tiles);              // [4 wavefronts][32 tokens][32 experts]
    float* mine = part + ((size_t)wave * 32 + ln) * 32;
#pragma unroll
    for (int g = 0; g < 4; g++)
        *reinterpret_cast<float4*>(mine + 8 * g + 4 * kb) = make_float4(acc[4 * g], acc[4 * g + 1], acc[4 * g + 2], acc[4 * g + 3]);
    __syncthreads();
    // thread: token tid / 8, experts 4 (tid % 8) .. + 3: 128 contiguous bytes of a row of the logits per 8 lanes
    const int tok = tid >> 3, ec = 4 * (tid & 7);
    if (t0 + tok < T) {
#pragma unroll
        for (int i = 0; i < 4; i++) {
            const int e = e0 + ec + i;
            if (e < E) {
                const int o = tok * 32 + ec + i;
                const float v = ((part[o] + part[1024 + o]) + part[2048 + o]) + part[3072 + o];
                logit[(size_t)(t0 + tok) * E + e] = v + (bias ? bias[e] : 0.0f);
            }
        }
    }
}

#ifndef DYMOE_RS_TB
#define DYMOE_RS_TB 1
#endif
constexpr int kRsBatch = DYMOE_RS_TB;      // tokens per wavefront
constexpr int kRsWaves = 4;
constexpr int kRsThreads = kRsWaves * kWave;

// Softmax and top-k from logits in memory.  The selection is a chain of cross-lane reductions, k rounds long, that one
// wavefront cannot overlap with anything but itself: what shortens the pass is more wavefronts, so each takes kRsBatch
// tokens only and reads their logits straight from memory (a lane holds every 64th expert).
__global__ __launch_bounds__(kRsThreads) void route_select_kernel(
    int T, int E, int k, int renorm, int32_t* __restrict__ idx, float* __restrict__ w,
    float* probs /* in: logits, out: probabilities */)
{
    extern __shared__ float smem[];                                  // [4 wavefronts][kRsBatch][k], used when k > 64
    const int wave = threadIdx.x / kWave;
    const int t0 = (blockIdx.x * kRsWaves + wave) * kRsBatch;
    if (t0 >= T) return;
    float* lgs[kRsBatch];
    float* sps[kRsBatch];
    int ts[kRsBatch];
#pragma unroll
    for (int b = 0; b < kRsBatch; b++) {
        const int t = min(t0 + b, T - 1);
        lgs[b] = probs + (size_t)t * E;
        sps[b] = smem + ((size_t)wave * kRsBatch + b) * k;
        ts[b] = (t0 + b < T) ? t0 + b : -1;
    }
    float* const (&lgc)[kRsBatch] = lgs;
    float* const (&spc)[kRsBatch] = sps;
    route_select_batch<kRsBatch>(lgc, spc, ts, E, k, renorm, idx, w, probs, nullptr, nullptr);
}

// Decode step front end in one workgroup: for each of the (few) tokens the
// gating of route_kernel<1, NCH, 8>, then the decode importance (mean gate
// probability, summed in token order), the load histogram and the ranked
// bit-width assignment, with the arithmetic of the stand-alone kernels.
template <int NCH, int NC>
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
        if (wave == 0) route_select_fixed<NC>(logit, selp, t, E, k, renorm, idx, w, probs, s_imp, s_load);
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
    assign_all<float>(8 * kWave, E, s_imp, s_load, tiers, floor_bits, bits, rank);
}

// The same front end for many experts, in two launches.  With 128 router rows of 2048 (512 KiB) one workgroup
// cannot keep enough loads in flight (a kilobyte per thread), so the logits take round after round of memory
// latency.  Here a wavefront owns one router row, kept in registers, and meets every token with it (the row is
// read once whatever T); the logits go to the probs buffer, and a single workgroup then does what is left.
//   logit[t, e] -> probs[t * E + e]      (overwritten with the probabilities by the second launch)
template <int NCH>
__global__ __launch_bounds__(8 * kWave) void front_logits_kernel(
    const uint16_t* __restrict__ x, const uint16_t* __restrict__ wg, const float* __restrict__ bias, int T, int H,
    int E, float* __restrict__ logit)
{
    const int lane = threadIdx.x & (kWave - 1);
    const int e = blockIdx.x * 8 + threadIdx.x / kWave;
    if (e >= E) return;
    const uint16_t* row = wg + (size_t)e * H;
    uint4 wv[NCH];
#pragma unroll
    for (int c = 0; c < NCH; c++) {
        wv[c] = make_uint4(0, 0, 0, 0);
        if (c * kWave * 8 < H) wv[c] = *reinterpret_cast<const uint4*>(row + min((c * kWave + lane) * 8, H - 8));
    }
    const float b = bias ? bias[e] : 0.0f;
    for (int t = 0; t < T; t++) {
        float acc = 0.0f;
#pragma unroll
        for (int c = 0; c < NCH; c++) {
            if (c * kWave * 8 < H) {  // uniform
                const int col = (c * kWave + lane) * 8;
                // lanes past the end meet the re-read tail of the row with zero activations
                uint4 xv = make_uint4(0, 0, 0, 0);
                if (col < H) xv = *reinterpret_cast<const uint4*>(x + (size_t)t * H + col);
                acc = dot2_bf16(wv[c].x, xv.x, acc);
                acc = dot2_bf16(wv[c].y, xv.y, acc);
                acc = dot2_bf16(wv[c].z, xv.z, acc);
                acc = dot2_bf16(wv[c].w, xv.w, acc);
            }
        }
        const float s = wave_sum(acc);
        if (lane == 0) logit[(size_t)t * E + e] = s + b;
    }
}

template <int NC>
__global__ __launch_bounds__(8 * kWave) void front_finish_kernel(
    int T, int E, int k, int renorm, int32_t* __restrict__ idx, float* __restrict__ w, float* __restrict__ probs,
    TierTable tiers, int floor_bits, float* __restrict__ importance, int32_t* __restrict__ load,
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
        __syncthreads();                            // the previous token's logits have been used
        for (int e = threadIdx.x; e < E; e += blockDim.x) logit[e] = probs[(size_t)t * E + e];
        __syncthreads();
        // tokens in order by one wavefront: the importance is a sum in token order
        if (wave == 0) route_select_fixed<NC>(logit, selp, t, E, k, renorm, idx, w, probs, s_imp, s_load);
    }
    __syncthreads();
    for (int e = threadIdx.x; e < E; e += blockDim.x) {
        const float g = s_imp[e];
        const float v = (T <= 1) ? g : g / (float)T;
        s_imp[e] = v;
        importance[e] = v;
        load[e] = s_load[e];
    }
    __syncthreads();
    assign_all<float>(8 * kWave, E, s_imp, s_load, tiers, floor_bits, bits, rank);
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

constexpr size_t kRouteMfmaMaxLds = 128 * 1024;

// Once per device, at context creation, with that device current: the matrix-core router asks for more dynamic LDS than
// the default limit (operand tiles, two partial tiles and the logits of 32 tokens).
int route_init()
{
    if (hipFuncSetAttribute(reinterpret_cast<const void*>(&route_mfma_kernel), hipFuncAttributeMaxDynamicSharedMemorySize,
                            (int)kRouteMfmaMaxLds) != hipSuccess)
        return DYMOE_EHIP;
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
    // many tokens and experts: a dense contraction, on the matrix cores (when its tiles fit in the LDS it may ask for)
    const size_t mfma_lds = (size_t)(dymoe::kRmTokens + dymoe::kRmExperts) * dymoe::kRmBK * 2 +
                            (2 * (size_t)dymoe::kRmTokens * dymoe::kRmExperts + (size_t)dymoe::kRmTokens * E +
                             (size_t)dymoe::kRmWaves * dymoe::kRmBatch * k) * sizeof(float);
    // few token tiles: cut by experts too and select in a second pass (the logits wait in the probs array)
    const int token_tiles = (T + dymoe::kRmTokens - 1) / dymoe::kRmTokens;
    const size_t select_lds = (size_t)dymoe::kRsWaves * dymoe::kRsBatch * k * sizeof(float);
    if (T >= 128 && E >= 64 && H % dymoe::kRlBK == 0 && probs && 2 * token_tiles <= ctx->num_cu) {
        dymoe_launch(ctx, DYMOE_K_ROUTE, dymoe::route_logits_kernel<dymoe::kRlBK>, dim3((unsigned)token_tiles, (unsigned)((E + 31) / 32)),
                     dim3(dymoe::kRlThreads), 0, st, (const uint16_t*)x, (const uint16_t*)wg, bias, T, H, E, probs);
        DYMOE_HIP_LAUNCH_CHECK();
        const int per_wg = dymoe::kRsWaves * dymoe::kRsBatch;
        dymoe_launch(ctx, DYMOE_K_ROUTE_SELECT, dymoe::route_select_kernel, dim3((unsigned)((T + per_wg - 1) / per_wg)),
                     dim3(dymoe::kRsThreads), select_lds, st, T, E, k, renorm, idx, w, probs);
        DYMOE_HIP_LAUNCH_CHECK();
        return DYMOE_OK;
    }
    if (T >= 128 && E >= 32 && H % 128 == 0 && mfma_lds <= dymoe::kRouteMfmaMaxLds) {
        dymoe_launch(ctx, DYMOE_K_ROUTE, dymoe::route_mfma_kernel, dim3((unsigned)((T + dymoe::kRmTokens - 1) / dymoe::kRmTokens)),
                     dim3(dymoe::kRmThreads), mfma_lds, st, (const uint16_t*)x, (const uint16_t*)wg, bias, T, H, E, k, renorm,
                     idx, w, probs);
        DYMOE_HIP_LAUNCH_CHECK();
        return DYMOE_OK;
    }
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
    // many experts (router of 256 KiB and more) and a probs buffer to pass the logits through: two launches
    if (probs && (size_t)E * (size_t)H * 2 >= ((size_t)256 << 10)) {
        const dim3 grid((unsigned)((E + 7) / 8));
        if (H <= 2048)
            dymoe_launch(ctx, DYMOE_K_ROUTE, (dymoe::front_logits_kernel<4>), grid, dim3(8 * dymoe::kWave), 0, st, xb, wb, bias,
                         T, H, E, probs);
        else if (H <= 4096)
            dymoe_launch(ctx, DYMOE_K_ROUTE, (dymoe::front_logits_kernel<8>), grid, dim3(8 * dymoe::kWave), 0, st, xb, wb, bias,
                         T, H, E, probs);
        else if (H <= 8192)
            dymoe_launch(ctx, DYMOE_K_ROUTE, (dymoe::front_logits_kernel<16>), grid, dim3(8 * dymoe::kWave), 0, st, xb, wb, bias,
                         T, H, E, probs);
        else
            dymoe_launch(ctx, DYMOE_K_ROUTE, (dymoe::front_logits_kernel<32>), grid, dim3(8 * dymoe::kWave), 0, st, xb, wb, bias,
                         T, H, E, probs);
        DYMOE_HIP_LAUNCH_CHECK();
#define DYMOE_FINISH(NC_)                                                                                              \
    dymoe_launch(ctx, DYMOE_K_DECODE_FRONT, (dymoe::front_finish_kernel<NC_>), dim3(1), dim3(8 * dymoe::kWave), smem, st, T, E, \
                 k, renorm, idx, w, probs, tt, floor_bits, importance, load, bits, rank)
        if (E <= 64) DYMOE_FINISH(1);
        else if (E <= 128) DYMOE_FINISH(2);
        else if (E <= 256) DYMOE_FINISH(4);
        else if (E <= 512) DYMOE_FINISH(8);
        else DYMOE_FINISH(16);
#undef DYMOE_FINISH
        DYMOE_HIP_LAUNCH_CHECK();
        return DYMOE_OK;
    }
#define DYMOE_FRONT(NCH_, NC_)                                                                                          \
    dymoe_launch(ctx, DYMOE_K_DECODE_FRONT, (dymoe::decode_front_kernel<NCH_, NC_>), dim3(1), dim3(8 * dymoe::kWave), smem, st, \
                 xb, wb, bias, T, H, E, k, renorm, idx, w, probs, tt, floor_bits, importance, load, bits, rank)
#define DYMOE_FRONT_BY_E(NCH_)                 \
    do {                                       \
        if (E <= 64) DYMOE_FRONT(NCH_, 1);     \
        else if (E <= 128) DYMOE_FRONT(NCH_, 2); \
        else if (E <= 256) DYMOE_FRONT(NCH_, 4); \
        else if (E <= 512) DYMOE_FRONT(NCH_, 8); \
        else DYMOE_FRONT(NCH_, 16);            \
    } while (0)
    if (H <= 4096) DYMOE_FRONT_BY_E(8);
    else if (H <= 8192) DYMOE_FRONT_BY_E(16);
    else DYMOE_FRONT_BY_E(32);
#undef DYMOE_FRONT_BY_E
#undef DYMOE_FRONT
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
