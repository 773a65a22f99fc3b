// Workspace layout of dymoe_moe_ffn_mixed (host side, shared by the size query
// and the two FFN paths).
#pragma once
#include <stddef.h>
#include <stdint.h>

namespace dymoe {

constexpr int kSeg = 2048;        // columns one wavefront covers per GEMV row segment
constexpr int kGemmTileM = 128;   // token rows per grouped-GEMM tile
constexpr int kGemmTileTall = 160; // the last tile of an int4 / int2 expert also takes a remainder of up to 32 rows
constexpr int kPlanTileMin = 32;  // sizing granularity of the tile list

struct FfnLayout {
    size_t hbuf;    // [P,F] SwiGLU intermediate: fp32 (GEMV) or 16-bit (GEMM)
    size_t part;    // GEMM: [P,H] fp32 per-pair outputs (the GEMV path keeps its partial sums on chip; the area is sized as before)
    size_t xh;      // GEMM: three [T,H] fp16 copies of the activations (int4 / int2 / natural column order)
    size_t plan;    // int32: counts[E], offsets[E+1], cursor[E], ntiles, perm[P], tiles[4*maxtiles], draft[4*maxtiles]
    size_t total;
    int max_tiles;
};

static inline size_t round256(size_t v) { return (v + 255) & ~(size_t)255; }

static inline FfnLayout ffn_layout(int T, int H, int F, int E, int k)
{
    FfnLayout L;
    size_t P = (size_t)T * (size_t)k;
    size_t nseg = ((size_t)F + kSeg - 1) / kSeg;
    L.max_tiles = (int)(P / kPlanTileMin + (size_t)E + 1);
    L.hbuf = 0;
    L.part = L.hbuf + round256(P * (size_t)F * 4);
    L.xh = L.part + round256(P * nseg * (size_t)H * 4);
    L.plan = L.xh + 3 * round256((size_t)T * (size_t)H * 2);
    size_t plan_ints = (size_t)E + ((size_t)E + 1) + (size_t)E + 8 + P + 8 * (size_t)L.max_tiles;
    L.total = L.plan + round256(plan_ints * 4);
    return L;
}

}  // namespace dymoe
