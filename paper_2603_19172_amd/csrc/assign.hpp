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
// s_imp / s_load: all E values (LDS).
template <typename ImpT>
__device__ __forceinline__ void assign_one(int e, int E, const ImpT* s_imp, const int32_t* s_load,
                                           const TierTable& tiers, int floor_bits,
                                           uint8_t* __restrict__ bits, int32_t* __restrict__ rank)
{
    const ImpT mi = s_imp[e];
    const int32_t ml = s_load[e];
    int pos = 0;
    // (unrolled so that the LDS reads of several experts are in flight together: one at a time, a read's
    // latency per expert made this loop the longest part of the step for 128 experts)
#pragma unroll 16
    for (int j = 0; j < E; j++) {
        const ImpT oi = s_imp[j];
        const int32_t ol = s_load[j];
        const bool first = (oi > mi) || (oi == mi && (ol > ml || (ol == ml && j < e)));
        pos += first ? 1 : 0;
    }
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

}  // namespace dymoe
