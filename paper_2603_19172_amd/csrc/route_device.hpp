// Device functions of the router gating shared by the routing kernels and the fused decode step: logits of a few
// tokens by a workgroup, softmax and top-k of a token by one wavefront.
#pragma once
#include <math.h>

#include "common.hpp"

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
    // A wavefront takes EB experts per round (all their rows requested before the first is used): with one token
    // the loop is nothing but memory latency, one round trip per round.
    constexpr int EB = (TW == 1) ? ((NCH <= 4) ? 4 : (NCH <= 8) ? 2 : 1) : 1;
    for (int e0 = wave; e0 < E; e0 += NW * EB) {
        uint4 wv[EB][NCH];
#pragma unroll
        for (int i = 0; i < EB; i++) {
            const int e = min(e0 + i * NW, E - 1);            // past the last expert: a copy of it, not stored
            const uint16_t* row = wg + (size_t)e * H;
#pragma unroll
            for (int c = 0; c < NCH; c++) {
                wv[i][c] = make_uint4(0, 0, 0, 0);
                if (c * kWave * 8 < H) {  // uniform
                    // lanes past the end re-read the row's tail against zero activations
                    const int col = min((c * kWave + lane) * 8, H - 8);
                    wv[i][c] = *reinterpret_cast<const uint4*>(row + col);
                }
            }
        }
#pragma unroll
        for (int i = 0; i < EB; i++) {
            const int e = e0 + i * NW;
            float acc[TW];
#pragma unroll
            for (int tw = 0; tw < TW; tw++) acc[tw] = 0.0f;
#pragma unroll
            for (int c = 0; c < NCH; c++) {
                if (c * kWave * 8 < H) {  // uniform
#pragma unroll
                    for (int tw = 0; tw < TW; tw++) {
                        acc[tw] = dot2_bf16(wv[i][c].x, xr[tw][c].x, acc[tw]);
                        acc[tw] = dot2_bf16(wv[i][c].y, xr[tw][c].y, acc[tw]);
                        acc[tw] = dot2_bf16(wv[i][c].z, xr[tw][c].z, acc[tw]);
                        acc[tw] = dot2_bf16(wv[i][c].w, xr[tw][c].w, acc[tw]);
                    }
                }
            }
            const float b = (bias && e < E) ? bias[e] : 0.0f;
#pragma unroll
            for (int tw = 0; tw < TW; tw++) {
                const float s = wave_sum(acc[tw]);
                if (lane == 0 && e < E) logit[tw * E + e] = s + b;
            }
        }
    }
}

// Softmax and top-k of TB tokens by one wavefront, from their logits in LDS.
// Lane l keeps the logits of experts l, l + 64, ... of every token in registers
// (NC per token, NC * 64 >= E); the k rounds of arg-max then run on registers
// alone: the largest remaining logit through the data-parallel primitives, the
// lowest expert index that holds it through a ballot, and the owner retires
// the entry.  The TB tokens are independent chains of the same arithmetic,
// written side by side so that their latencies overlap; every token's result
// is what TB = 1 gives.
// t[b] < 0: token b is padding (computed, nothing written to global memory).
// selp[b]: k floats of LDS scratch per token.  prob_sum (LDS, may be null):
// prob_sum[e] += p[e]; load_cnt (LDS, may be null): load_cnt[e] += 1 for the
// selected experts.
template <int TB, int NC>
__device__ __forceinline__ void route_select_regs(float* const (&lg)[TB], float* const (&selp)[TB],
                                                  const int (&t)[TB], int E, int k, int renorm,
                                                  int32_t* __restrict__ idx, float* __restrict__ w,
                                                  float* probs, float* prob_sum,
                                                  int32_t* load_cnt)
{
    const int lane = threadIdx.x & (kWave - 1);
    float v[TB][NC];
    float mx[TB], den[TB], rden[TB], sel_sum[TB], mine[TB];
#pragma unroll
    for (int b = 0; b < TB; b++) mine[b] = 0.0f;
#pragma unroll
    for (int b = 0; b < TB; b++) {
        mx[b] = -INFINITY;
#pragma unroll
        for (int c = 0; c < NC; c++) {
            const int e = c * kWave + lane;
            v[b][c] = (e < E) ? lg[b][e] : -INFINITY;
            mx[b] = fmaxf(mx[b], v[b][c]);
        }
    }
#pragma unroll
    for (int b = 0; b < TB; b++) {
        mx[b] = wave_max_dpp(mx[b]);
        den[b] = 0.0f;
#pragma unroll
        for (int c = 0; c < NC; c++)
            if (c * kWave + lane < E) den[b] += expf(v[b][c] - mx[b]);
    }
#pragma unroll
    for (int b = 0; b < TB; b++) {
        den[b] = wave_sum_dpp(den[b]);
        rden[b] = 1.0f / den[b];
        sel_sum[b] = 0.0f;
    }
    if (probs || prob_sum) {
#pragma unroll
        for (int b = 0; b < TB; b++)
#pragma unroll
            for (int c = 0; c < NC; c++) {
                const int e = c * kWave + lane;
                if (e < E && t[b] >= 0) {
                    const float p = expf(v[b][c] - mx[b]) * rden[b];
                    if (probs) probs[(size_t)t[b] * E + e] = p;
                    if (prob_sum) prob_sum[e] += p;
                }
            }
    }
    for (int j = 0; j < k; j++) {
#pragma unroll
        for (int b = 0; b < TB; b++) {
            // the largest remaining logit, then the lowest expert index that holds it
            float bv = v[b][0];
#pragma unroll
            for (int c = 1; c < NC; c++) bv = fmaxf(bv, v[b][c]);
            bv = wave_max_dpp(bv);
            int bi = -1;
#pragma unroll
            for (int c = 0; c < NC; c++) {
                const unsigned long long hit = __ballot(c * kWave + lane < E && v[b][c] == bv);
                if (bi < 0 && hit) bi = c * kWave + __ffsll((long long)hit) - 1;
            }
            const float p = expf(bv - mx[b]) * rden[b];      // the same in every lane
            sel_sum[b] += p;
            if (k <= kWave) {
                if (lane == j) mine[b] = p;                   // lane j keeps the j-th gate weight
            } else if (lane == 0) {
                selp[b][j] = p;
            }
            if (lane == 0) {
                if (t[b] >= 0) idx[(size_t)t[b] * k + j] = bi;
                if (load_cnt && t[b] >= 0) load_cnt[bi] += 1;
            }
#pragma unroll
            for (int c = 0; c < NC; c++)
                if (c * kWave + lane == bi) v[b][c] = -INFINITY;        // the owner retires the entry
        }
    }
    if (k <= kWave) {
        // up to 64 selected experts: the weights never leave the registers (no LDS hand-over, and so no wait for
        // the stores above, which the fences of the other branch imply)
#pragma unroll
        for (int b = 0; b < TB; b++) {
            const float scale = renorm ? 1.0f / sel_sum[b] : 1.0f;
            if (t[b] >= 0 && lane < k) w[(size_t)t[b] * k + lane] = mine[b] * scale;
        }
        return;
    }
    __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "wavefront");      // selp: written by lane 0, read by all
    __builtin_amdgcn_wave_barrier();
#pragma unroll
    for (int b = 0; b < TB; b++) {
        const float scale = renorm ? 1.0f / sel_sum[b] : 1.0f;
        if (t[b] >= 0)
            for (int j = lane; j < k; j += kWave) w[(size_t)t[b] * k + j] = selp[b][j] * scale;
    }
    __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "wavefront");
    __builtin_amdgcn_wave_barrier();
}

// one token, the number of logits per lane fixed by the caller (E <= 64 NC): the single-workgroup front-end
// kernels are launched once per step with cold instruction caches, and every select variant they carry but do
// not run is code they still have to fetch past
template <int NC>
__device__ __forceinline__ void route_select_fixed(float* lg, float* selp, int t, int E, int k, int renorm,
                                                   int32_t* __restrict__ idx, float* __restrict__ w,
                                                   float* probs, float* prob_sum, int32_t* load_cnt)
{
    float* const lgs[1] = {lg};
    float* const sps[1] = {selp};
    const int ts[1] = {t};
    route_select_regs<1, NC>(lgs, sps, ts, E, k, renorm, idx, w, probs, prob_sum, load_cnt);
}

}  // namespace dymoe
