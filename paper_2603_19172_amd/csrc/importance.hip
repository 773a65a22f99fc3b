// Expert importance (heavy-hitter token load / gate score) and the
// importance-ranked bit-width assignment.  Both are tiny: integer histograms
// and an E x E ranking, sized for one or a few workgroups.
#include <math.h>

#include "common.hpp"
#include "assign.hpp"

namespace dymoe {

constexpr int kImpThreads = 1024;

// zero-fill without hipMemsetAsync (the calls may be captured into a graph)
__global__ void zero_i32_kernel(int32_t* a, int32_t* b, int n)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) {
        a[i] = 0;
        if (b) b[i] = 0;
    }
}

// Prefill: a token is a heavy hitter when fewer than k_hh tokens precede it in
// the order (score descending, token index ascending).  kImpLanes adjacent
// lanes share one token: all T scores pass through LDS, 2048 per trip (a
// thread's two requested together), each lane compares the token against its
// share of every 1024 of them (four scores per read), and the partial counts
// are added across the lanes.  (32 lanes per token and 1024 threads: with 8
// lanes and 256 threads the 2048 tokens of the 128-expert layer kept 256
// wavefronts busy on a chip of 1024 SIMDs, a memory latency per 256 scores,
// and four times as many workgroups queued up at the E global counters.)  The token's first lane
// then adds its k routed experts to the workgroup's LDS histograms (load and,
// if heavy, importance); the workgroup adds its non-zero bins to the global
// ones, which the caller has zeroed.  with_importance = 0: only the load
// histogram (decode).
constexpr int kImpLanes = 32;
constexpr int kImpTokens = kImpThreads / kImpLanes;      // tokens per workgroup
constexpr int kImpStage = 2 * kImpThreads;               // scores in LDS per trip

__global__ __launch_bounds__(kImpThreads) void importance_prefill_kernel(
    const int32_t* __restrict__ idx, const float* __restrict__ score, int T, int E, int k,
    int k_hh, int with_importance, int32_t* __restrict__ importance, int32_t* __restrict__ load)
{
    __shared__ __attribute__((aligned(16))) float tile[kImpStage];
    __shared__ int32_t s_load[DYMOE_MAX_EXPERTS];
    __shared__ int32_t s_imp[DYMOE_MAX_EXPERTS];
    for (int e = threadIdx.x; e < E; e += kImpThreads) {
        s_load[e] = 0;
        s_imp[e] = 0;
    }
    const int part = threadIdx.x % kImpLanes;
    const int t = blockIdx.x * kImpTokens + threadIdx.x / kImpLanes;
    bool heavy = false;
    if (with_importance) {
        const float mine = (t < T) ? score[t] : 0.0f;
        int before = 0;
        constexpr int kSpan = kImpThreads / kImpLanes;     // scores of a tile that one lane looks at
        for (int base = 0; base < T; base += kImpStage) {
            // a thread's eight scores of this trip are requested together (one at a time, every 256 scores cost a
            // memory latency: eight of them for the 2048 tokens of the 128-expert layer)
            float v[kImpStage / kImpThreads];
#pragma unroll
            for (int u = 0; u < kImpStage / kImpThreads; u++) {
                const int i = base + u * kImpThreads + (int)threadIdx.x;
                // slots past the end hold -inf at an index past every token: never counted
                v[u] = (i < T) ? score[i] : -INFINITY;
            }
            __syncthreads();                               // the previous trip's scores have been read
#pragma unroll
            for (int u = 0; u < kImpStage / kImpThreads; u++) tile[u * kImpThreads + threadIdx.x] = v[u];
            __syncthreads();
            const int pieces = min(kImpStage / kImpThreads, (T - base + kImpThreads - 1) / kImpThreads);
            for (int piece = 0; piece < pieces; piece++) {
#pragma unroll
                for (int j = part * kSpan; j < (part + 1) * kSpan; j += 4) {
                    const float4 s4 = *reinterpret_cast<const float4*>(tile + piece * kImpThreads + j);
                    const int u0 = base + piece * kImpThreads + j;
                    before += (s4.x > mine || (s4.x == mine && u0 + 0 < t)) ? 1 : 0;
                    before += (s4.y > mine || (s4.y == mine && u0 + 1 < t)) ? 1 : 0;
                    before += (s4.z > mine || (s4.z == mine && u0 + 2 < t)) ? 1 : 0;
                    before += (s4.w > mine || (s4.w == mine && u0 + 3 < t)) ? 1 : 0;
                }
            }
        }
#pragma unroll
        for (int o = 1; o < kImpLanes; o <<= 1) before += __shfl_xor(before, o, kWave);
        heavy = (t < T) && before < k_hh;
    } else {
        __syncthreads();
    }
    if (t < T && part == 0) {
        for (int s = 0; s < k; s++) {
            const int e = idx[(size_t)t * k + s];
            if (e < 0 || e >= E) continue;
            atomicAdd(&s_load[e], 1);
            if (heavy) atomicAdd(&s_imp[e], 1);
        }
    }
    __syncthreads();
    for (int e = threadIdx.x; e < E; e += kImpThreads) {
        if (s_load[e]) atomicAdd(&load[e], s_load[e]);
        if (with_importance && s_imp[e]) atomicAdd(&importance[e], s_imp[e]);
    }
}

// Single-workgroup version of both phases for short steps (decode, a few
// tokens): histograms live in LDS, so there is nothing to zero beforehand and
// the whole step is one launch.
constexpr int kImpBlock = 1024;

__global__ __launch_bounds__(kImpBlock) void importance_block_kernel(
    const int32_t* __restrict__ idx, const float* __restrict__ score,
    const float* __restrict__ probs, int T, int E, int k, int k_hh, int prefill,
    void* __restrict__ importance, int32_t* __restrict__ load)
{
    __shared__ int32_t s_load[DYMOE_MAX_EXPERTS];
    __shared__ int32_t s_imp[DYMOE_MAX_EXPERTS];
    __shared__ float tile[kImpBlock];
    const int tid = threadIdx.x;
    for (int e = tid; e < E; e += kImpBlock) {
        s_load[e] = 0;
        s_imp[e] = 0;
    }
    __syncthreads();
    const int chunks = (T + kImpBlock - 1) / kImpBlock;   // same trip count for every thread
    for (int c = 0; c < chunks; c++) {
        const int t = c * kImpBlock + tid;
        bool heavy = false;
        if (prefill) {
            const float mine = (t < T) ? score[t] : 0.0f;
            int before = 0;
            for (int b = 0; b < chunks; b++) {
                const int u = b * kImpBlock + tid;
                tile[tid] = (u < T) ? score[u] : 0.0f;
                __syncthreads();
                const int n = min(kImpBlock, T - b * kImpBlock);
                for (int j = 0; j < n; j++) {
                    const float s = tile[j];
                    before += (s > mine || (s == mine && b * kImpBlock + j < t)) ? 1 : 0;
                }
                __syncthreads();
            }
            heavy = (t < T) && before < k_hh;
        }
        if (t < T) {
            for (int s = 0; s < k; s++) {
                const int e = idx[(size_t)t * k + s];
                if (e < 0 || e >= E) continue;
                atomicAdd(&s_load[e], 1);
                if (heavy) atomicAdd(&s_imp[e], 1);
            }
        }
    }
    __syncthreads();
    for (int e = tid; e < E; e += kImpBlock) {
        load[e] = s_load[e];
        if (prefill) {
            reinterpret_cast<int32_t*>(importance)[e] = s_imp[e];
        } else {
            float g = 0.0f;
            for (int t = 0; t < T; t++) g += probs[(size_t)t * E + e];
            reinterpret_cast<float*>(importance)[e] = (T <= 1) ? g : g / (float)T;
        }
    }
}

// Decode: importance[e] = mean over the step's tokens of the gate score
__global__ void importance_decode_kernel(const float* __restrict__ probs, int T, int E,
                                         float* __restrict__ importance)
{
    const int e = blockIdx.x * blockDim.x + threadIdx.x;
    if (e >= E) return;
    float s = 0.0f;
    for (int t = 0; t < T; t++) s += probs[(size_t)t * E + e];
    importance[e] = (T == 1) ? s : s / (float)T;
}

// One workgroup of 1024 threads: up to eight lanes share an expert's ranking.
template <typename ImpT>
__global__ __launch_bounds__(DYMOE_MAX_EXPERTS) void assign_precision_kernel(
    const ImpT* __restrict__ importance, const int32_t* __restrict__ load, int E, TierTable tiers,
    int floor_bits, uint8_t* __restrict__ bits, int32_t* __restrict__ rank)
{
    __shared__ ImpT s_imp[DYMOE_MAX_EXPERTS];
    __shared__ int32_t s_load[DYMOE_MAX_EXPERTS];
    for (int e = threadIdx.x; e < E; e += blockDim.x) {
        s_imp[e] = importance[e];
        s_load[e] = load ? load[e] : 0;
    }
    __syncthreads();
    assign_all<ImpT>((int)blockDim.x, E, s_imp, s_load, tiers, floor_bits, bits, rank);
}

}  // namespace dymoe

extern "C" {

int dymoe_expert_importance(dymoe_ctx* ctx, int phase, const int32_t* idx, const float* probs,
                            const float* token_score, int T, int E, int k, int k_hh,
                            void* importance, int32_t* load, void* stream)
{
    DYMOE_REQUIRE(importance && load);
    DYMOE_REQUIRE(phase == DYMOE_PHASE_PREFILL || phase == DYMOE_PHASE_DECODE);
    DYMOE_REQUIRE(T >= 0 && E > 0 && k > 0 && k <= E);
    if (phase == DYMOE_PHASE_PREFILL) DYMOE_REQUIRE(k_hh >= 0 && k_hh <= T);
    if (T > 0) {
        DYMOE_REQUIRE(idx != nullptr);
        if (phase == DYMOE_PHASE_PREFILL) DYMOE_REQUIRE(token_score != nullptr);
        else DYMOE_REQUIRE(probs != nullptr);
    }
    if (E > DYMOE_MAX_EXPERTS) return DYMOE_ENOTSUP;
    if (!ctx) return DYMOE_ENOCTX;
    hipStream_t st = (hipStream_t)stream;
    const bool prefill = phase == DYMOE_PHASE_PREFILL;
    // one workgroup ranks T tokens against T scores, a thread per token walking all T: one launch, but 3.5 us at 16
    // tokens, 7.8 at 64 and 24 at 256, against 5.5-6 us for the zero-fill and the many-workgroup kernel behind it
    if (T <= 32) {
        dymoe_launch(ctx, DYMOE_K_IMPORTANCE, dymoe::importance_block_kernel, dim3(1),
                     dim3(dymoe::kImpBlock), 0, st, idx, token_score, probs, T, E, k, k_hh,
                     prefill ? 1 : 0, importance, load);
        DYMOE_HIP_LAUNCH_CHECK();
        return DYMOE_OK;
    }
    hipLaunchKernelGGL(dymoe::zero_i32_kernel, dim3((E + 255) / 256), dim3(256), 0, st, load,
                       prefill ? (int32_t*)importance : (int32_t*)nullptr, E);
    DYMOE_HIP_LAUNCH_CHECK();
    if (T > 0) {
        const unsigned blocks = (unsigned)((T + dymoe::kImpTokens - 1) / dymoe::kImpTokens);
        dymoe_launch(ctx, DYMOE_K_IMPORTANCE, dymoe::importance_prefill_kernel, dim3(blocks), dim3(dymoe::kImpThreads),
                           0, st, idx, token_score, T, E, k, k_hh, prefill ? 1 : 0,
                           (int32_t*)importance, load);
        DYMOE_HIP_LAUNCH_CHECK();
    }
    if (!prefill) {
        hipLaunchKernelGGL(dymoe::importance_decode_kernel, dim3((E + 255) / 256), dim3(256), 0, st,
                           probs, T, E, (float*)importance);
        DYMOE_HIP_LAUNCH_CHECK();
    }
    return DYMOE_OK;
}

int dymoe_assign_precision(dymoe_ctx* ctx, int phase, const void* importance,
                           const int32_t* load, int E, int n_tiers,
                           const int32_t* tier_count, const uint8_t* tier_bits, int floor_bits,
                           uint8_t* bits, int32_t* rank, void* stream)
{
    DYMOE_REQUIRE(importance && tier_count && tier_bits && bits);
    DYMOE_REQUIRE(phase == DYMOE_PHASE_PREFILL || phase == DYMOE_PHASE_DECODE);
    DYMOE_REQUIRE(E > 0 && n_tiers >= 1 && n_tiers <= DYMOE_MAX_TIERS);
    DYMOE_REQUIRE(floor_bits == 0 || floor_bits == 2 || floor_bits == 4 || floor_bits == 8 || floor_bits == 16);
    dymoe::TierTable tt;
    DYMOE_REQUIRE(dymoe::make_tier_table(E, n_tiers, tier_count, tier_bits, tt) == DYMOE_OK);
    if (E > DYMOE_MAX_EXPERTS) return DYMOE_ENOTSUP;
    if (!ctx) return DYMOE_ENOCTX;
    hipStream_t st = (hipStream_t)stream;
    // enough threads for eight lanes per expert, at most the 1024 of a workgroup
    unsigned threads = (unsigned)(((E * 8 + 63) / 64) * 64);
    if (threads > DYMOE_MAX_EXPERTS) threads = DYMOE_MAX_EXPERTS;
    if (phase == DYMOE_PHASE_PREFILL)
        dymoe_launch(ctx, DYMOE_K_ASSIGN, (dymoe::assign_precision_kernel<int32_t>), dim3(1), dim3(threads), 0, st,
                           (const int32_t*)importance, load, E, tt, floor_bits, bits, rank);
    else
        dymoe_launch(ctx, DYMOE_K_ASSIGN, (dymoe::assign_precision_kernel<float>), dim3(1), dim3(threads), 0, st,
                           (const float*)importance, load, E, tt, floor_bits, bits, rank);
    DYMOE_HIP_LAUNCH_CHECK();
    return DYMOE_OK;
}

}  // extern "C"
