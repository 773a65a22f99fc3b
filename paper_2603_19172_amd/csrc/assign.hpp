// The ranked bit-width assignment of one expert, shared by the stand-alone
// assignment kernel and the fused decode front end.
#pragma once
#include "common.hpp"

namespace dymoe {

struct TierTable {
    int n;
    int32_t count[DYMOE_MAX_TIERS];
    uint8_t bits[DYMOE_MAX_TIERS];
};

// Host side: check and copy the caller's tier arrays.  Returns DYMOE_OK or DYMOE_EINVAL.
inline int make_tier_table(int E, int n_tiers, const int32_t* tier_count, const uint8_t* tier_bits,
                           TierTable& tt)
{
    if (!tier_count || !tier_bits || n_tiers < 1 || n_tiers > DYMOE_MAX_TIERS) return DYMOE_EINVAL;
    tt.n = n_tiers;
    long total = 0;
    for (int i = 0; i < DYMOE_MAX_TIERS; i++) {
        tt.count[i] = 0;
        tt.bits[i] = 0;
    }
    for (int i = 0; i < n_tiers; i++) {
        const int b = tier_bits[i];
        if (tier_count[i] < 0) return DYMOE_EINVAL;
        if (!(b == 0 || b == 2 || b == 4 || b == 8 || b == 16)) return DYMOE_EINVAL;
        tt.count[i] = tier_count[i];
        tt.bits[i] = (uint8_t)b;
        total += tier_count[i];
    }
    return total == E ? DYMOE_OK : DYMOE_EINVAL;
}

// Expert e counts the experts that precede it in the order (importance
// descending, load descending, index ascending) -> rank -> tier -> bits.
// s_imp / s_load: all E values (LDS).  S adjacent lanes share an expert (S a
// power of two up to 8, lane = e * S + part): each counts every S-th rival and
// the counts are added across the S lanes; the lane with part 0 writes.  All
// lanes of a wavefront must call (the cross-lane sum has no branches around it);
// a lane whose e is past the end passes e >= E and writes nothing.
template <typename ImpT, int S>
__device__ __forceinline__ void assign_shared(int e, int part, int E, const ImpT* s_imp, const int32_t* s_load,
                                              const TierTable& tiers, int floor_bits,
                                              uint8_t* __restrict__ bits, int32_t* __restrict__ rank)
{
    const int me = min(e, E - 1);
    const ImpT mi = s_imp[me];
    const int32_t ml = s_load[me];
    int pos = 0;
    // (unrolled so that the LDS reads of several rivals are in flight together)
#pragma unroll 8
    for (int j = part; j < E; j += S) {
        const ImpT oi = s_imp[j];
        const int32_t ol = s_load[j];
        const bool first = (oi > mi) || (oi == mi && (ol > ml || (ol == ml && j < me)));
        pos += first ? 1 : 0;
    }
#pragma unroll
    for (int o = 1; o < S; o <<= 1) pos += __shfl_xor(pos, o, kWave);
    if (e >= E || part != 0) return;
    int tier = 0, upto = tiers.count[0];
    while (pos >= upto && tier + 1 < tiers.n) {
        tier++;
        upto += tiers.count[tier];
    }
    int b = tiers.bits[tier];
    if (b < floor_bits) b = floor_bits;
    bits[e] = (uint8_t)b;
    if (rank) rank[e] = pos;
}

// All experts by a workgroup of `threads` threads (a multiple of 64; every thread must call).
template <typename ImpT>
__device__ __forceinline__ void assign_all(int threads, int E, const ImpT* s_imp, const int32_t* s_load,
                                           const TierTable& tiers, int floor_bits,
                                           uint8_t* __restrict__ bits, int32_t* __restrict__ rank)
{
    const int tid = threadIdx.x;
    if (E * 8 <= threads) {
        assign_shared<ImpT, 8>(tid >> 3, tid & 7, E, s_imp, s_load, tiers, floor_bits, bits, rank);
    } else if (E * 4 <= threads) {
        assign_shared<ImpT, 4>(tid >> 2, tid & 3, E, s_imp, s_load, tiers, floor_bits, bits, rank);
    } else if (E * 2 <= threads) {
        assign_shared<ImpT, 2>(tid >> 1, tid & 1, E, s_imp, s_load, tiers, floor_bits, bits, rank);
    } else {
        for (int e0 = 0; e0 < E; e0 += threads)
            assign_shared<ImpT, 1>(e0 + tid, 0, E, s_imp, s_load, tiers, floor_bits, bits, rank);
    }
}

}  // namespace dymoe
