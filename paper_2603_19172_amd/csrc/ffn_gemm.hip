// Prefill path of the mixed-precision SwiGLU expert FFN: tokens grouped by
// expert, one MFMA grouped GEMM per projection, all experts in one launch.
//
// Work unit: up to 128 token rows of one expert x (4 wavefronts x 2 strips of
// 32 weight rows), K walked in tiles of 128.
//  * Weights never touch LDS.  They are stored in 32 x 128 tiles whose byte
//    order is the MFMA A-operand order (lane (r, kb) owns row r, columns
//    64 kb .. 64 kb + 64, one quantisation group), so every load instruction of
//    a wavefront reads 1 KiB of contiguous memory straight into the registers
//    the MFMA consumes (bf16) or the dequantiser consumes (int4 / int2).
//  * The token tile is shared by the 4 wavefronts through a double-buffered
//    LDS tile; it is copied from a 16-bit copy of the activations that is
//    already in the column order the code fields come out of a dword, so
//    staging is a plain copy: global memory -> LDS directly
//    (global_load_lds_dwordx4), stored swizzled so that the operand reads are
//    free of bank conflicts without padding.
//  * bf16 experts: v_mfma_f32_32x32x16_bf16 on the bf16 activations.
//    int4 / int2 experts: v_mfma_f32_32x32x16_f16 on an fp16 copy of the
//    activations; weights become fp16 in registers: a code field OR-ed into the
//    mantissa of 2^n (n such that the field's lowest bit weighs one) is the
//    number 2^n + q; subtracting 2^n is exact; then one packed fma(q, s, m).
//  * A workgroup is four wavefronts, one per SIMD, and two workgroups share a
//    compute unit: the two wavefronts of a SIMD belong to different workgroups,
//    so one's barrier, waits, prologue and epilogue are covered by the other's
//    MFMA work.
//  * Results leave through LDS: in the MFMA result layout a lane holds a few
//    outputs of one token's row, so stores made from it would touch 32 rows per
//    instruction; the token-tile buffers, free after the K loop, turn the
//    rows round so that 16 lanes store 256 contiguous bytes of one row.
#include <math.h>

#include "common.hpp"
#include "ffn_layout.hpp"

namespace dymoe {

constexpr int kGmThreads = 256;
constexpr int kGmWaves = 4;         // one per SIMD; two workgroups share a compute unit
constexpr int kBK = 128;            // K-tile
constexpr int kXsBufBytes = kGemmTileTall * kBK * 2;   // one token tile in LDS: up to 160 rows x 256 bytes, no padding

// Tiles of one expert with c pairs at b bits: 128 rows each, the last one shorter.  For the int4 and int2 formats a
// last remainder of 1..32 rows is attached to the tile before it instead (5 fragments of 32 tokens, 160 rows): a
// remainder tile streams and dequantises the expert's whole weight matrices once more for a handful of tokens, which
// costs a third to a half of a full tile's time and all of its memory traffic.  (bf16 and int8 strips leave no
// registers for a fifth pair of accumulators.)
__device__ __forceinline__ bool plan_tall(int c, int b)
{
    const int r = c % kGemmTileM;
    return (b == 4 || b == 2) && c > kGemmTileM && r >= 1 && r <= kGemmTileTall - kGemmTileM;
}
__device__ __forceinline__ int plan_tiles_of(int c, int b)
{
    return (c + kGemmTileM - 1) / kGemmTileM - (plan_tall(c, b) ? 1 : 0);
}

// ----------------------------------------------------------------------------
// plan: counting sort of the (token, slot) pairs by expert + tile list
// ints: counts[E] | offsets[E+1] | cursor[E] | ntiles (8 ints) | perm[P] | tiles[4*max_tiles] | draft[4*max_tiles]
// (cursor: its first E BYTES hold the bit width every expert is run at, which is bits[e] unless the table lacks that
// format, then 0; the GEMM and combine kernels read these instead of bits[])
struct PlanPtrs {
    int32_t* counts;
    int32_t* offsets;
    int32_t* cursor;
    int32_t* ntiles;
    int32_t* perm;
    int32_t* tiles;
};

__host__ __device__ inline PlanPtrs plan_ptrs(int32_t* base, int E, int P)
{
    PlanPtrs p;
    p.counts = base;
    p.offsets = p.counts + E;
    p.cursor = p.offsets + E + 1;
    p.ntiles = p.cursor + E;
    p.perm = p.ntiles + 8;
    p.tiles = p.perm + P;
    return p;
}

// One workgroup of 16 wavefronts.  Counting and scattering go through one
// histogram per wavefront when they fit in LDS (E <= kPlanPrivE), so that the
// atomics of a popular expert do not queue up across the whole workgroup; a
// pair's position is then (expert offset) + (pairs of the expert in earlier
// wavefronts) + (its turn inside its wavefront).  Tiles are laid out by one
// thread per expert after a scan of the per-expert tile counts, staged in LDS
// when the list fits, and sorted by rank counting.
constexpr int kPlanThreads = 1024;
constexpr int kPlanWaves = kPlanThreads / kWave;
constexpr int kPlanPrivE = 256;        // 16 x 256 counters = 16 KiB
constexpr int kPlanLdsTiles = 1024;    // 4 ints each = 16 KiB
constexpr int kPlanRankStrides = 4;    // tile lists of up to 4 x 64 entries are ranked from registers

__global__ __launch_bounds__(kPlanThreads) void plan_kernel(const int32_t* __restrict__ idx,
                                                            const uint8_t* __restrict__ bits,
                                                            const dymoe_expert_fmt* __restrict__ table, int P, int E,
                                                            int tile_m, int max_tiles,
                                                            int32_t* __restrict__ plan, unsigned* __restrict__ flags)
{
    __shared__ int32_t s_count[DYMOE_MAX_EXPERTS];
    __shared__ int32_t s_off[DYMOE_MAX_EXPERTS + 1];
    __shared__ int32_t s_tile0[DYMOE_MAX_EXPERTS + 1];       // first tile of each expert
    __shared__ int32_t s_priv[kPlanWaves * kPlanPrivE];
    __shared__ __attribute__((aligned(16))) int32_t s_draft[4 * kPlanLdsTiles];
    __shared__ uint8_t s_bits[DYMOE_MAX_EXPERTS];
    const PlanPtrs pp = plan_ptrs(plan, E, P);
    const int tid = threadIdx.x, wave = tid / kWave;
    const bool priv = E <= kPlanPrivE;
    for (int e = tid; e < E; e += kPlanThreads) {
        s_count[e] = 0;
        int b = bits[e];
        if (b == 16 || b == 8 || b == 4 || b == 2) {
            // a format the table does not hold: the expert is left out, as at 0 bits.  Whether it had pairs is not
            // known yet, but the decode path reports the same condition only for routed experts: checked below.
            if (!dymoe_fmt_present(table[e], b)) b = 0x80 | b;
        } else {
            b = 0;
        }
        s_bits[e] = (uint8_t)b;
    }
    if (priv)
        for (int i = tid; i < kPlanWaves * E; i += kPlanThreads) s_priv[i] = 0;
    __syncthreads();
    // (the expert indices of a batch of pairs are requested together and looked at afterwards: one pair at a time, every
    // iteration waited a memory latency for its own index, 16 latencies per pass on the 128-expert layer)
    constexpr int kPlanBatch = 16;
    // up to 16 x 1024 pairs: a thread's indices stay in registers from the counting pass to the scattering pass
    const bool one_pass = P <= kPlanBatch * kPlanThreads;
    int es[kPlanBatch];
    auto counted = [&](int e) {
        if (e < 0 || e >= E) return false;
        const int b = s_bits[e];
        if (b & 0x80) {                       // routed to, selected format absent: say so, leave the pair out
            atomicOr(flags, DYMOE_FLAG_FORMAT_MISSING);
            return false;
        }
        return b != 0;
    };
    for (int p0 = tid; p0 < P || p0 == tid; p0 += kPlanBatch * kPlanThreads) {
#pragma unroll
        for (int u = 0; u < kPlanBatch; u++) {
            const int p = p0 + u * kPlanThreads;
            es[u] = (p < P) ? idx[p] : -1;
        }
#pragma unroll
        for (int u = 0; u < kPlanBatch; u++)
            if (counted(es[u])) atomicAdd(priv ? &s_priv[wave * E + es[u]] : &s_count[es[u]], 1);
    }
    __syncthreads();
    if (priv) {
        // per expert: total, and every wavefront's first position among the expert's pairs
        for (int e = tid; e < E; e += kPlanThreads) {
            int run = 0;
            for (int wv = 0; wv < kPlanWaves; wv++) {
                const int c = s_priv[wv * E + e];
                s_priv[wv * E + e] = run;
                run += c;
            }
            s_count[e] = run;
        }
        __syncthreads();
    }
    // exclusive scans over the experts (pairs and tiles): E is at most 1024, one wavefront walks it in strides
    if (wave == 0) {
        const int lane = tid;
        int run = 0, trun = 0, with_tiles = 0;
        for (int e0 = 0; e0 < E; e0 += kWave) {
            const int e = e0 + lane;
            const int c = (e < E) ? s_count[e] : 0;
            const int nt_e = (e < E) ? plan_tiles_of(c, s_bits[e]) : 0;
            int incl = c, tincl = nt_e;
#pragma unroll
            for (int o = 1; o < kWave; o <<= 1) {
                const int a = __shfl_up(incl, o, kWave), b2 = __shfl_up(tincl, o, kWave);
                if (lane >= o) {
                    incl += a;
                    tincl += b2;
                }
            }
            if (e < E) {
                s_off[e] = run + incl - c;
                s_tile0[e] = trun + tincl - nt_e;
            }
            run += __shfl(incl, kWave - 1, kWave);
            trun += __shfl(tincl, kWave - 1, kWave);
            with_tiles += __popcll(__ballot(nt_e > 0));
        }
        if (lane == 0) {
            s_off[E] = run;
            s_tile0[E] = trun;
            pp.ntiles[0] = trun;
            pp.ntiles[1] = run;
            pp.ntiles[2] = with_tiles;      // experts with at least one tile (the GEMM launches pick their XCD mapping by it)
        }
    }
    __syncthreads();
    const int nt_all = s_tile0[E];
    // (written once for a draft in LDS and once for a draft in memory, so that neither is reached through flat accesses)
    auto lay_out_and_rank = [&](int32_t* draft) {
        for (int e = tid; e < E; e += kPlanThreads) {
            const int c = s_count[e], b = s_bits[e];
            int nt = s_tile0[e];
            const int nt_end = nt + plan_tiles_of(c, b);
            for (int m0 = 0; nt < nt_end; m0 += tile_m, nt++) {
                const int rows = (nt == nt_end - 1) ? c - m0 : tile_m;     // (the last tile: up to 160 rows when tall)
                draft[4 * nt + 0] = e;
                draft[4 * nt + 1] = s_off[e] + m0;
                draft[4 * nt + 2] = rows;
                // cost key, roughly the time a workgroup spends on the tile: streaming (bf16)
                // or dequantising (int4, int2) the weights costs the same whatever the number
                // of tokens; the MFMA work grows with the 32-token fragments
                draft[4 * nt + 3] = (b == 16 ? 100 : (b == 2 ? 60 : 61)) + 10 * ((rows + 31) >> 5);
            }
        }
        __syncthreads();        // (workgroup-wide visibility also of the draft kept in global memory)
        // Longest first: workgroups are dispatched in tile order, so the cheap tiles
        // (few tokens) fill the end of the launch instead of stretching it.
        // Rank by counting, (key descending, position ascending): a permutation.
        // A wavefront per tile: its lanes share the comparisons against all tiles (one thread per tile walked the
        // whole list alone, a dependent LDS read per step: 9 us for the 174 tiles of the 128-expert layer).
        const int lane = tid & (kWave - 1);
        if (nt_all <= kPlanRankStrides * kWave) {
            // up to 256 tiles: a lane keeps the keys of tiles lane, 64 + lane, ... in registers, counts on the vector
            // unit and the counts meet through DPP: a trip of the loop is one LDS read long (with the keys re-read
            // and a ballot per stride counted on the scalar unit a trip was a chain of five dependent LDS reads and
            // as many vector-to-scalar hand-overs: 8.2 us for the 197 tiles of the 128-expert layer)
            int keys[kPlanRankStrides];
#pragma unroll
            for (int u = 0; u < kPlanRankStrides; u++) {
                const int j = u * kWave + lane;
                keys[u] = (j < nt_all) ? draft[4 * j + 3] : -1;          // (-1: below every key)
            }
            for (int i = wave; i < nt_all; i += kPlanWaves) {
                const int rec = draft[4 * i + (lane & 3)];
                const int key = __builtin_amdgcn_readlane(rec, 3);
                int cnt = 0;
#pragma unroll
                for (int u = 0; u < kPlanRankStrides; u++) {
                    const int j = u * kWave + lane;
                    cnt += (keys[u] > key || (keys[u] == key && j < i)) ? 1 : 0;
                }
                const int pos = wave_sum_dpp_i32(cnt);
                if (lane < 4) pp.tiles[4 * pos + lane] = rec;
            }
        } else {
            for (int i = wave; i < nt_all; i += kPlanWaves) {
                const int key = draft[4 * i + 3];
                int pos = 0;        // the same in every lane: each stride of 64 tiles adds the number of its lanes that precede i
                for (int j0 = 0; j0 < nt_all; j0 += kWave) {
                    const int j = j0 + lane;
                    const int kj = (j < nt_all) ? draft[4 * j + 3] : -1;
                    pos += __popcll(__ballot(j < nt_all && (kj > key || (kj == key && j < i))));
                }
                if (lane < 4) pp.tiles[4 * pos + lane] = draft[4 * i + lane];
            }
        }
    };
    if (max_tiles <= kPlanLdsTiles) lay_out_and_rank(s_draft);
    else lay_out_and_rank(pp.tiles + 4 * (size_t)max_tiles);
    for (int e = tid; e < E; e += kPlanThreads) {
        pp.counts[e] = s_count[e];
        pp.offsets[e] = s_off[e];
        reinterpret_cast<uint8_t*>(pp.cursor)[e] = (s_bits[e] & 0x80) ? 0 : s_bits[e];
    }
    if (tid == 0) pp.offsets[E] = s_off[E];
    __syncthreads();
    for (int e = tid; e < E; e += kPlanThreads) s_count[e] = 0;    // reused as the scatter cursor
    __syncthreads();
    // order inside an expert is arbitrary: every row of a tile is computed independently
    for (int p0 = tid; p0 < P || p0 == tid; p0 += kPlanBatch * kPlanThreads) {
        if (!one_pass) {
#pragma unroll
            for (int u = 0; u < kPlanBatch; u++) {
                const int p = p0 + u * kPlanThreads;
                es[u] = (p < P) ? idx[p] : -1;
            }
        }
#pragma unroll
        for (int u = 0; u < kPlanBatch; u++) {
            const int e = es[u];
            if (!counted(e)) continue;
            const int pos = s_off[e] + (priv ? atomicAdd(&s_priv[wave * E + e], 1) : atomicAdd(&s_count[e], 1));
            pp.perm[pos] = p0 + u * kPlanThreads;
        }
    }
}

// Column order in which the code fields of a dword come out of the mask-and-or
// extraction: inside every 8 columns (int4) 0,4,1,5,2,6,3,7; inside every 16
// columns (int2) 0,8,1,9,...,7,15.  Inputs are packed pairs of 16-bit values.
__device__ __forceinline__ uint4 perm8(const uint4 v)
{
    uint4 o;
    o.x = (v.x & 0xffffu) | (v.z << 16);
    o.y = (v.x >> 16) | (v.z & 0xffff0000u);
    o.z = (v.y & 0xffffu) | (v.w << 16);
    o.w = (v.y >> 16) | (v.w & 0xffff0000u);
    return o;
}

__device__ __forceinline__ void perm16(const uint4 a, const uint4 b, uint4& o0, uint4& o1)
{
    o0.x = (a.x & 0xffffu) | (b.x << 16);
    o0.y = (a.x >> 16) | (b.x & 0xffff0000u);
    o0.z = (a.y & 0xffffu) | (b.y << 16);
    o0.w = (a.y >> 16) | (b.y & 0xffff0000u);
    o1.x = (a.z & 0xffffu) | (b.z << 16);
    o1.y = (a.z >> 16) | (b.z & 0xffff0000u);
    o1.z = (a.w & 0xffffu) | (b.w << 16);
    o1.w = (a.w >> 16) | (b.w & 0xffff0000u);
}

// Three fp16 copies of the bf16 activations (exact inside fp16's normal range):
// one in each of the column orders above and one in the natural order (int8
// codes come out of a dword in order).  A thread converts 16 columns.
__global__ __launch_bounds__(256) void prep_x_kernel(const uint16_t* __restrict__ x, long n16,
                                                     uint16_t* __restrict__ xh4,
                                                     uint16_t* __restrict__ xh2,
                                                     uint16_t* __restrict__ xh8)
{
    const long i = (long)blockIdx.x * 256 + threadIdx.x;
    if (i >= n16) return;
    const uint4 a = reinterpret_cast<const uint4*>(x)[2 * i];
    const uint4 b = reinterpret_cast<const uint4*>(x)[2 * i + 1];
    uint4 ha, hb;
    ha.x = pack_half2(bf16_lo(a.x), bf16_hi(a.x)); ha.y = pack_half2(bf16_lo(a.y), bf16_hi(a.y));
    ha.z = pack_half2(bf16_lo(a.z), bf16_hi(a.z)); ha.w = pack_half2(bf16_lo(a.w), bf16_hi(a.w));
    hb.x = pack_half2(bf16_lo(b.x), bf16_hi(b.x)); hb.y = pack_half2(bf16_lo(b.y), bf16_hi(b.y));
    hb.z = pack_half2(bf16_lo(b.z), bf16_hi(b.z)); hb.w = pack_half2(bf16_lo(b.w), bf16_hi(b.w));
    reinterpret_cast<uint4*>(xh4)[2 * i] = perm8(ha);
    reinterpret_cast<uint4*>(xh4)[2 * i + 1] = perm8(hb);
    uint4 o0, o1;
    perm16(ha, hb, o0, o1);
    reinterpret_cast<uint4*>(xh2)[2 * i] = o0;
    reinterpret_cast<uint4*>(xh2)[2 * i + 1] = o1;
    reinterpret_cast<uint4*>(xh8)[2 * i] = ha;
    reinterpret_cast<uint4*>(xh8)[2 * i + 1] = hb;
}

// ----------------------------------------------------------------------------
// weight strips (32 rows x one K-tile of 128), as one lane holds them

template <int BITS> struct StripRaw;
template <> struct StripRaw<16> { uint4 r[8]; };
template <> struct StripRaw<8> { uint4 r[4]; uint32_t s2, m2; };
template <> struct StripRaw<4> { uint4 r[2]; uint32_t s2, m2; };
template <> struct StripRaw<2> { uint4 r[1]; uint32_t s2, m2; };

struct MatPtr {
    const uint16_t* w;    // bf16 row-major
    const char* wt;       // bf16 tiles (may be null)
    const char* q;        // packed codes, tile layout
    const uint16_t* s;    // fp16 scale, tile layout
    const uint16_t* z;    // fp16 zero, tile layout
};

__device__ __forceinline__ MatPtr mat_ptr(const dymoe_expert_fmt& ex, int mat, int b)
{
    MatPtr m;
    m.w = reinterpret_cast<const uint16_t*>(ex.w[mat]);
    m.wt = reinterpret_cast<const char*>(ex.wt[mat]);
    m.q = reinterpret_cast<const char*>((b == 8) ? ex.q8[mat] : (b == 4) ? ex.q4[mat] : ex.q2[mat]);
    m.s = reinterpret_cast<const uint16_t*>((b == 8) ? ex.s8[mat] : (b == 4) ? ex.s4[mat] : ex.s2[mat]);
    m.z = reinterpret_cast<const uint16_t*>((b == 8) ? ex.z8[mat] : (b == 4) ? ex.z4[mat] : ex.z2[mat]);
    return m;
}

__device__ __forceinline__ uint32_t deq_pair(uint32_t biased, uint32_t bias2, uint32_t s2, uint32_t m2)
{
    const half2_t q = __builtin_bit_cast(half2_t, biased) - __builtin_bit_cast(half2_t, bias2);  // exact
    const half2_t r = __builtin_elementwise_fma(q, __builtin_bit_cast(half2_t, s2),
                                                __builtin_bit_cast(half2_t, m2));
    return __builtin_bit_cast(uint32_t, r);
}

// A fragments of MFMA sub-steps 2*jj and 2*jj+1 (8 k each) of one strip
template <int BITS>
__device__ __forceinline__ void strip_frags(const StripRaw<BITS>& raw, int jj, uint4& f0, uint4& f1)
{
    if constexpr (BITS == 16) {
        f0 = raw.r[2 * jj];
        f1 = raw.r[2 * jj + 1];
    } else if constexpr (BITS == 8) {
        // 16 codes, one per byte, in k order: a byte b becomes the fp16 number 1024 + b
        const uint4 q = raw.r[jj];
        f0.x = deq_pair(__builtin_amdgcn_perm(0x64646464u, q.x, 0x04010400u), 0x64006400u, raw.s2, raw.m2);
        f0.y = deq_pair(__builtin_amdgcn_perm(0x64646464u, q.x, 0x04030402u), 0x64006400u, raw.s2, raw.m2);
        f0.z = deq_pair(__builtin_amdgcn_perm(0x64646464u, q.y, 0x04010400u), 0x64006400u, raw.s2, raw.m2);
        f0.w = deq_pair(__builtin_amdgcn_perm(0x64646464u, q.y, 0x04030402u), 0x64006400u, raw.s2, raw.m2);
        f1.x = deq_pair(__builtin_amdgcn_perm(0x64646464u, q.z, 0x04010400u), 0x64006400u, raw.s2, raw.m2);
        f1.y = deq_pair(__builtin_amdgcn_perm(0x64646464u, q.z, 0x04030402u), 0x64006400u, raw.s2, raw.m2);
        f1.z = deq_pair(__builtin_amdgcn_perm(0x64646464u, q.w, 0x04010400u), 0x64006400u, raw.s2, raw.m2);
        f1.w = deq_pair(__builtin_amdgcn_perm(0x64646464u, q.w, 0x04030402u), 0x64006400u, raw.s2, raw.m2);
    } else if constexpr (BITS == 4) {
        const uint4 q = raw.r[jj >> 1];
        const uint32_t w0 = (jj & 1) ? q.z : q.x;
        const uint32_t w1 = (jj & 1) ? q.w : q.y;
        // k order inside a fragment: 0,4,1,5,2,6,3,7
        uint32_t v = w0, v8 = w0 >> 8;
        f0.x = deq_pair(and_or(v, 0x000F000Fu, 0x64006400u), 0x64006400u, raw.s2, raw.m2);
        f0.y = deq_pair(and_or(v, 0x00F000F0u, 0x54005400u), 0x54005400u, raw.s2, raw.m2);
        f0.z = deq_pair(and_or(v8, 0x000F000Fu, 0x64006400u), 0x64006400u, raw.s2, raw.m2);
        f0.w = deq_pair(and_or(v8, 0x00F000F0u, 0x54005400u), 0x54005400u, raw.s2, raw.m2);
        v = w1; v8 = w1 >> 8;
        f1.x = deq_pair(and_or(v, 0x000F000Fu, 0x64006400u), 0x64006400u, raw.s2, raw.m2);
        f1.y = deq_pair(and_or(v, 0x00F000F0u, 0x54005400u), 0x54005400u, raw.s2, raw.m2);
        f1.z = deq_pair(and_or(v8, 0x000F000Fu, 0x64006400u), 0x64006400u, raw.s2, raw.m2);
        f1.w = deq_pair(and_or(v8, 0x00F000F0u, 0x54005400u), 0x54005400u, raw.s2, raw.m2);
    } else {
        const uint4 q = raw.r[0];
        const uint32_t v = (jj == 0) ? q.x : (jj == 1) ? q.y : (jj == 2) ? q.z : q.w;
        const uint32_t v10 = v >> 10;
        // 16 codes of the dword; k order 0,8,1,9,2,10,3,11 | 4,12,5,13,6,14,7,15
        f0.x = deq_pair(and_or(v, 0x00030003u, 0x64006400u), 0x64006400u, raw.s2, raw.m2);
        f0.y = deq_pair(and_or(v, 0x000C000Cu, 0x5C005C00u), 0x5C005C00u, raw.s2, raw.m2);
        f0.z = deq_pair(and_or(v, 0x00300030u, 0x54005400u), 0x54005400u, raw.s2, raw.m2);
        f0.w = deq_pair(and_or(v, 0x00C000C0u, 0x4C004C00u), 0x4C004C00u, raw.s2, raw.m2);
        f1.x = deq_pair(and_or(v, 0x03000300u, 0x44004400u), 0x44004400u, raw.s2, raw.m2);
        f1.y = deq_pair(and_or(v10, 0x00030003u, 0x64006400u), 0x64006400u, raw.s2, raw.m2);
        f1.z = deq_pair(and_or(v10, 0x000C000Cu, 0x5C005C00u), 0x5C005C00u, raw.s2, raw.m2);
        f1.w = deq_pair(and_or(v10, 0x00300030u, 0x54005400u), 0x54005400u, raw.s2, raw.m2);
    }
}

template <int BITS>
__device__ __forceinline__ float16_t mfma16(const uint4 a, const uint4 b, const float16_t c)
{
    if constexpr (BITS == 16)
        return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, a),
                                                      __builtin_bit_cast(bf16x8_t, b), c, 0, 0, 0);
    else
        return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(half8_t, a),
                                                      __builtin_bit_cast(half8_t, b), c, 0, 0, 0);
}

// address of this lane's slice of the K-tiles of one 32-row strip
struct StripSrc {
    const char* p;        // this lane's first 16 bytes of K-tile 0 (bf16 tiles or rows, or packed codes)
    const uint16_t* s;    // scale / zero at this lane's slot of K-tile 0 (quantised only)
    const uint16_t* z;
    int kt_stride;        // bytes from one K-tile to the next
    int c_stride;         // bytes from one 16-byte chunk of the lane's slice to the next
};

template <int BITS>
__device__ __forceinline__ StripSrc strip_src(const MatPtr& m, long nt, int K, int lane)
{
    StripSrc src;
    const long tile_row = nt * (K >> 7);
    src.s = m.s + tile_row * 64 + (uint32_t)lane;
    src.z = m.z + tile_row * 64 + (uint32_t)lane;
    if constexpr (BITS == 16) {
        if (m.wt) {          // tiles: chunk c of every lane sits in one 1 KiB run
            src.p = m.wt + tile_row * 8192 + (uint32_t)(lane * 16);
            src.kt_stride = 8192;
            src.c_stride = 1024;
        } else {             // rows: the lane's 64 columns are contiguous
            src.p = reinterpret_cast<const char*>(m.w + (nt * 32 + (lane & 31)) * K + 64 * (lane >> 5));
            src.kt_stride = 256;
            src.c_stride = 16;
        }
    } else {
        src.p = m.q + tile_row * (512 * BITS) + (uint32_t)(lane * 16);      // 32 x 128 codes of BITS bits: 512 * BITS bytes per tile
        src.kt_stride = 512 * BITS;
        src.c_stride = 1024;
    }
    return src;
}

// chunk c of the lane's slice of K-tile kt: bf16 c = 0..7 (8 columns each),
// int8 c = 0..3 (16 codes each), int4 c = 0..1 (32 codes each), int2 c = 0 (64 codes)
template <int BITS>
__device__ __forceinline__ uint4 load_chunk(const StripSrc& src, int kt, int c)
{
    if constexpr (BITS == 16) return load_global<uint4>(src.p + (long)kt * src.kt_stride + c * src.c_stride);
    else if constexpr (BITS == 8) return load_global<uint4>(src.p + (long)kt * 4096 + c * 1024);
    else if constexpr (BITS == 4) return load_global<uint4>(src.p + (long)kt * 2048 + c * 1024);
    else return load_global<uint4>(src.p + (long)kt * 1024);
}

template <int BITS>
__device__ __forceinline__ void load_scale_zero(const StripSrc& src, int kt, StripRaw<BITS>& raw)
{
    if constexpr (BITS != 16) {
        // the 16-bit values as loaded; adopt_strip() duplicates them into both halves
        raw.s2 = load_global<uint16_t>(src.s + kt * 64);
        raw.m2 = load_global<uint16_t>(src.z + kt * 64);
    }
}

// Make a freshly loaded strip the current one.  Touching the loaded values is
// left to this point, a whole K-tile after the request, so nothing waits for a
// load right after issuing it.
template <int BITS>
__device__ __forceinline__ void adopt_strip(StripRaw<BITS>& cur, const StripRaw<BITS>& next)
{
    cur = next;
    if constexpr (BITS != 16) {
        cur.s2 |= cur.s2 << 16;
        cur.m2 |= cur.m2 << 16;
    }
}

template <int BITS>
__device__ __forceinline__ void load_strip(const StripSrc& src, int kt, StripRaw<BITS>& raw)
{
    constexpr int kChunks = (BITS == 16) ? 8 : (BITS == 8 ? 4 : (BITS == 4 ? 2 : 1));
#pragma unroll
    for (int c = 0; c < kChunks; c++) raw.r[c] = load_chunk<BITS>(src, kt, c);
    load_scale_zero<BITS>(src, kt, raw);
}

// 16 bytes of LDS at a byte address
__device__ __forceinline__ uint4 lds_read16(uint32_t addr)
{
    const u32x4_t v = *(const __attribute__((address_space(3))) u32x4_t*)(uintptr_t)addr;
    return __builtin_bit_cast(uint4, v);
}

__device__ __forceinline__ void lds_write16(uint32_t addr, const uint4 v)
{
    *(__attribute__((address_space(3))) u32x4_t*)(uintptr_t)addr = __builtin_bit_cast(u32x4_t, v);
}

typedef uint32_t u32x2_t __attribute__((ext_vector_type(2)));

__device__ __forceinline__ void lds_write8(uint32_t addr, const uint2 v)
{
    *(__attribute__((address_space(3))) u32x2_t*)(uintptr_t)addr = __builtin_bit_cast(u32x2_t, v);
}

__device__ __forceinline__ uint32_t lds_read4(uint32_t addr)
{
    return *(const __attribute__((address_space(3))) uint32_t*)(uintptr_t)addr;
}

__device__ __forceinline__ void lds_write4(uint32_t addr, uint32_t v)
{
    *(__attribute__((address_space(3))) uint32_t*)(uintptr_t)addr = v;
}

// second GEMM's epilogue: a wavefront's own LDS area, 32 rows of 256 bytes + 16 of padding
constexpr uint32_t kEpiRowBytes = 272;
constexpr uint32_t kEpiWaveBytes = 32 * kEpiRowBytes;
static_assert(kGmWaves * kEpiWaveBytes <= (uint32_t)kXsBufBytes, "the epilogue areas fit in the first token-tile buffer");
static_assert(kGemmTileTall * kEpiRowBytes <= 2 * (uint32_t)kXsBufBytes, "the first GEMM's output rows fit in the two buffers");

// The token operands of one MFMA step (two 16-byte chunks of one row).
struct XOps {
    uint4 t0, t1;
};

// Quarters JJ0 .. JJ1-1 of one K-tile of MFMAs for NTF token fragments (32 tokens each).
// A step is one (quarter, fragment) pair: four MFMAs on two LDS chunks.  The
// chunks of step s+1 are requested before the MFMAs of step s are issued, so the
// LDS latency hides behind arithmetic; the operands of a tile's first step come
// in through `ops`.  Scheduling barriers keep this order.
// bf16 (64 registers of raw weights per K-tile): the loads of the next K-tile
// are woven into the sequence; every weight register is refilled as soon as
// the last MFMA that reads it has been issued, so the next tile's weights are
// in flight during three quarters of this tile's arithmetic without a second
// set of registers.
// int8 (16 registers of codes per strip): refilled in place like bf16; only the
// scale and zero of the next tile wait in registers of their own.
// int4 / int2 (10 / 6 registers per strip): the next tile's codes were already
// requested into a second register set before this call; nothing to load here.
template <int BITS, int NTF, int JJ0, int JJ1>
__device__ __forceinline__ void compute_ktile(StripRaw<BITS>& ra, StripRaw<BITS>& rb,
                                              const StripSrc& sa, const StripSrc& sb, int kt_next,
                                              uint32_t xa, XOps& ops, float16_t (&acc)[2][NTF])
{
    constexpr int kStepMask = 0x2 | 0x4;            // VALU and SALU may cross; MFMA, LDS and global accesses may not
#pragma unroll
    for (int jj = JJ0; jj < JJ1; jj++) {
        uint4 a0, a1, b0, b1;
        strip_frags<BITS>(ra, jj, a0, a1);
        strip_frags<BITS>(rb, jj, b0, b1);
#pragma unroll
        for (int tf = 0; tf < NTF; tf++) {
            if constexpr (NTF == 5) {
                // five fragments: 160 accumulator registers leave no room for a second pair of operands, so a step
                // reads its own (the other wavefront of the SIMD covers the LDS latency)
                const uint32_t x0 = (xa ^ (uint32_t)(jj << 5)) + tf * (32 * kBK * 2);
                ops.t0 = lds_read16(x0);
                ops.t1 = lds_read16(x0 ^ 16u);
                __builtin_amdgcn_sched_barrier(kStepMask);
                acc[0][tf] = mfma16<BITS>(a0, ops.t0, acc[0][tf]);
                acc[1][tf] = mfma16<BITS>(b0, ops.t0, acc[1][tf]);
                acc[0][tf] = mfma16<BITS>(a1, ops.t1, acc[0][tf]);
                acc[1][tf] = mfma16<BITS>(b1, ops.t1, acc[1][tf]);
                __builtin_amdgcn_sched_barrier(kStepMask);
            } else {
            // next step: next fragment, else next quarter (nothing after the tile's last step)
            const bool wrap = (tf == NTF - 1);
            const bool last = wrap && jj == 3;
            const int njj = wrap ? jj + 1 : jj;
            const int ntf = wrap ? 0 : tf + 1;
            XOps nxt = ops;
            if (!last) {
                const uint32_t x0 = (xa ^ (uint32_t)(njj << 5)) + ntf * (32 * kBK * 2);
                nxt.t0 = lds_read16(x0);
                nxt.t1 = lds_read16(x0 ^ 16u);
            }
            __builtin_amdgcn_sched_barrier(kStepMask);
            acc[0][tf] = mfma16<BITS>(a0, ops.t0, acc[0][tf]);
            acc[1][tf] = mfma16<BITS>(b0, ops.t0, acc[1][tf]);
            acc[0][tf] = mfma16<BITS>(a1, ops.t1, acc[0][tf]);
            acc[1][tf] = mfma16<BITS>(b1, ops.t1, acc[1][tf]);
            ops = nxt;
            __builtin_amdgcn_sched_barrier(kStepMask);
            }
        }
        if constexpr (BITS == 16) {
            ra.r[2 * jj] = load_chunk<16>(sa, kt_next, 2 * jj);
            ra.r[2 * jj + 1] = load_chunk<16>(sa, kt_next, 2 * jj + 1);
            rb.r[2 * jj] = load_chunk<16>(sb, kt_next, 2 * jj);
            rb.r[2 * jj + 1] = load_chunk<16>(sb, kt_next, 2 * jj + 1);
            __builtin_amdgcn_sched_barrier(kStepMask);
        } else if constexpr (BITS == 8) {
            ra.r[jj] = load_chunk<8>(sa, kt_next, jj);
            rb.r[jj] = load_chunk<8>(sb, kt_next, jj);
            __builtin_amdgcn_sched_barrier(kStepMask);
        } else if constexpr (NTF == 5 && BITS == 4) {
            // five fragments: no second register set; each 16-byte chunk of codes serves two quarters and is
            // refilled when the second is done, half a tile before the next tile needs it
            if (jj & 1) {
                ra.r[jj >> 1] = load_chunk<4>(sa, kt_next, jj >> 1);
                rb.r[jj >> 1] = load_chunk<4>(sb, kt_next, jj >> 1);
                __builtin_amdgcn_sched_barrier(kStepMask);
            }
        }
    }
}

// Global-memory instructions issued per K-tile after the token-tile copies
// (every one of them unconditional): the copies are older than all of them, so
// "at most this many memory operations still in flight" means the copies landed.
template <int BITS>
constexpr int ktile_loads()
{
    return BITS == 16 ? 16 : (BITS == 8 ? 12 : (BITS == 4 ? 8 : 6));
}

// ----------------------------------------------------------------------------
// Token tile: global memory -> LDS without passing through registers.
//
// global_load_lds_dwordx4 writes the 16 bytes a lane fetched to
// LDS[M0 + 16 * lane]: one instruction fills 1 KiB = 4 tile rows of 256 bytes.
// The lane chooses WHAT it fetches, so the tile is stored swizzled for free:
// row r keeps its 16-byte chunk c at chunk position c ^ (r & 15).  The MFMA
// operand reads (lane = row, fixed c) then fall on 16 different chunk
// positions for 16 consecutive rows, i.e. on all banks once.
// Wavefront w fills rows 32 i + 4 w .. + 3 (i = 0 .. NTF-1); a thread's rows
// all have the same r & 15, hence the same source chunk.
// The instruction is issued from inline assembly so that the compiler does not
// make every later LDS read wait for it; completion is awaited explicitly
// (wait_tile_copies) before the workgroup barrier that publishes the tile.
__device__ __forceinline__ void lds_copy16(const char* base, uint32_t lane_offset, uint32_t lds_addr_lane0)
{
    // base is the same for the whole wavefront (scalar registers), lane_offset an unsigned 32-bit byte offset
    asm volatile("s_mov_b32 m0, %0\n\tglobal_load_lds_dwordx4 %1, %2"
                 :
                 : "s"(lds_addr_lane0), "v"(lane_offset), "s"(base)
                 : "memory");
}

template <int N>
__device__ __forceinline__ void wait_tile_copies()
{
    static_assert(N >= 0 && N < 64, "vmcnt is a 6-bit counter");
    asm volatile("s_waitcnt vmcnt(%0)" : : "n"(N) : "memory");
    // the same wait once more in a form the compiler's own bookkeeping reads
    // (vmcnt = N, no wait on the export and LDS/scalar counters): it then knows
    // that older loads have completed and does not wait for them again later,
    // when such a wait would also cover copies issued in between
    __builtin_amdgcn_s_waitcnt(0x0F70 | (N & 15) | ((N >> 4) << 14));
}

constexpr int kRowsPerCopy = 4 * kGmWaves;      // tile rows the workgroup fills with one instruction per wavefront

template <int NTF>
struct XStage {
    static constexpr int kCopies = 32 * NTF / kRowsPerCopy;
    const char* base;            // start of the activation matrix (the same in every lane)
    uint32_t off[kCopies];       // byte offset of this thread's 16 bytes of K-tile 0 in each of its rows
    uint32_t lds;                // LDS address of lane 0's slot of the wavefront's first unit, buffer 0
};

template <int NTF>
__device__ __forceinline__ void copy_tile(const XStage<NTF>& st, int kt, int buf)
{
    const char* base = st.base + (long)kt * (kBK * 2);
#pragma unroll
    for (int i = 0; i < XStage<NTF>::kCopies; i++)
        lds_copy16(base, st.off[i], st.lds + buf * kXsBufBytes + i * (kRowsPerCopy * kBK * 2));
}

// ----------------------------------------------------------------------------
// MODE 1: h = silu(x W1^T) * (x W3^T)   strips = (W1 rows, W3 rows) of the same 32 features
// MODE 2: o = h W2^T                     strips = two adjacent groups of 32 rows of W2,
//                                        K-tiles [kt_begin, kt_end) of the split
template <int MODE, int BITS, int NTF>
__device__ __forceinline__ void gemm_tile(
    const uint16_t* __restrict__ act,   // MODE 1: [T,K] activations (gathered); MODE 2: [P,K] intermediate
    const int32_t* __restrict__ perm, int k_route, const dymoe_expert_fmt& ex, int K, int N,
    int kt_begin, int kt_end, int row0, int rows, int nblock, uint16_t* __restrict__ hout,
    float* __restrict__ oout, uint32_t xs_base)
{
    const int tid = threadIdx.x;
    const int lane = tid & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(tid / kWave);     // (the same in every lane: addresses built from it stay scalar)
    const int ln = lane & 31;
    const int kb = lane >> 5;

    // strips of this wavefront (32-row tiles of the weight matrices)
    long nt_a, nt_b;
    MatPtr ma, mb;
    bool strip_ok[2];
    if (MODE == 1) {
        nt_a = nt_b = (long)nblock * kGmWaves + wave;
        ma = mat_ptr(ex, 0, BITS);
        mb = mat_ptr(ex, 1, BITS);
        strip_ok[0] = strip_ok[1] = nt_a * 32 < N;
    } else {
        nt_a = ((long)nblock * kGmWaves + wave) * 2;
        nt_b = nt_a + 1;
        ma = mb = mat_ptr(ex, 2, BITS);
        strip_ok[0] = nt_a * 32 < N;
        strip_ok[1] = nt_b * 32 < N;
    }
    if (!strip_ok[0]) nt_a = 0;   // idle strips stream tile row 0; their results are dropped
    if (!strip_ok[1]) nt_b = 0;

    float16_t acc[2][NTF];
#pragma unroll
    for (int s = 0; s < 2; s++)
#pragma unroll
        for (int tf = 0; tf < NTF; tf++)
#pragma unroll
            for (int i = 0; i < 16; i++) acc[s][tf][i] = 0.0f;

    // staging role: rows 16 i + 4 wave + lane / 16, physical chunk lane % 16.
    // Tile rows past the expert's last token re-read its last token: their
    // products are computed and dropped, and the loop stays branch-free.
    XStage<NTF> stage;
    {
        const int rb = 4 * wave + (lane >> 4);
        const int chunk = (lane & 15) ^ (rb & 15);
#pragma unroll
        for (int i = 0; i < XStage<NTF>::kCopies; i++) {
            const int r = min(kRowsPerCopy * i + rb, rows - 1);
            const long src_row = (MODE == 1) ? (long)(perm[row0 + r] / k_route) : (long)(row0 + r);
            stage.off[i] = (uint32_t)(src_row * K * 2 + 16 * chunk);     // < 4 GiB, checked by the launcher
        }
        stage.base = reinterpret_cast<const char*>(act);
        stage.lds = __builtin_amdgcn_readfirstlane(xs_base + wave * 1024);
    }
    // operand reads: lane (ln, kb) reads row 32 tf + ln, chunks 8 kb + 2 jj (+1)
    const uint32_t xa0 = xs_base + ln * (kBK * 2) + (((uint32_t)kb << 7) ^ ((uint32_t)(ln & 15) << 4));
    uint32_t xa = xa0;

    // K loop over two LDS buffers: the next token tile is copied into the other
    // buffer while this one is multiplied.  The two workgroups of a compute unit
    // run independently, so one's barrier, prologue and epilogue overlap the
    // other's arithmetic.
    const StripSrc sa = strip_src<BITS>(ma, nt_a, K, lane);
    const StripSrc sb = strip_src<BITS>(mb, nt_b, K, lane);
    StripRaw<BITS> ra, rb;
    copy_tile<NTF>(stage, kt_begin, 0);
    load_strip<BITS>(sa, kt_begin, ra);
    load_strip<BITS>(sb, kt_begin, rb);
    adopt_strip<BITS>(ra, ra);
    adopt_strip<BITS>(rb, rb);
    wait_tile_copies<0>();
    __syncthreads();
    int buf = 0;          // buffer of tile kt
    for (int kt = kt_begin; kt < kt_end; kt++) {
        // past the end the prefetches re-read the last tile instead of branching
        const int kn = min(kt + 1, kt_end - 1);
        copy_tile<NTF>(stage, kn, buf ^ 1);
        StripRaw<BITS> na, nb;
        constexpr bool kSecondSet = (BITS == 2) || (BITS == 4 && NTF != 5);    // next tile's codes in registers of their own
        if constexpr (kSecondSet) {
            load_strip<BITS>(sa, kn, na);
            load_strip<BITS>(sb, kn, nb);
            __builtin_amdgcn_sched_barrier(0);   // keep the requests up here, a whole tile ahead of their use
        }
        XOps ops;             // operands of the first step
        ops.t0 = lds_read16(xa);
        ops.t1 = lds_read16(xa ^ 16u);
        if constexpr (BITS == 8 || (BITS == 4 && NTF == 5)) {
            // the next tile's scale and zero are requested after the first quarter's
            // refills: a wait for a refilled register then never reaches back to
            // the copies issued at the top of the tile before a quarter has passed
            compute_ktile<BITS, NTF, 0, 1>(ra, rb, sa, sb, kn, xa, ops, acc);
            load_scale_zero<BITS>(sa, kn, na);
            load_scale_zero<BITS>(sb, kn, nb);
            __builtin_amdgcn_sched_barrier(0);
            compute_ktile<BITS, NTF, 1, 4>(ra, rb, sa, sb, kn, xa, ops, acc);
            ra.s2 = na.s2 | (na.s2 << 16);
            ra.m2 = na.m2 | (na.m2 << 16);
            rb.s2 = nb.s2 | (nb.s2 << 16);
            rb.m2 = nb.m2 | (nb.m2 << 16);
            __builtin_amdgcn_sched_barrier(0);
        } else {
            compute_ktile<BITS, NTF, 0, 4>(ra, rb, sa, sb, kn, xa, ops, acc);
        }
        if constexpr (kSecondSet) {
            adopt_strip<BITS>(ra, na);
            adopt_strip<BITS>(rb, nb);
            // finish the hand-over here, not after the next tile's requests
            // (a wait placed there would also wait for the copies just issued)
            __builtin_amdgcn_sched_barrier(0);
        }
        wait_tile_copies<ktile_loads<BITS>()>();
        __syncthreads();
        buf ^= 1;
        xa = xa0 + (uint32_t)(buf * kXsBufBytes);
    }

    // epilogue.  D layout: lane (ln, kb), register i -> weight row 8*(i/4) + 4*kb + i%4, token ln
    if constexpr (MODE == 2) {
        // Down projection: a lane holds, of its token's row, 4 consecutive outputs per register group: stored as they
        // are, one instruction would touch 32 rows with 32 bytes each.  The wavefront turns each fragment round in LDS
        // instead (the token tiles are done with: the loop's last barrier follows the last tile's arithmetic and the
        // last copy's wait): 32 rows of its 64 columns, 256 bytes + 16 of padding per row (the padding keeps both the
        // lane-per-row writes and the 16-lanes-per-row reads free of bank conflicts, and holds the row's pair index),
        // read back so that 16 lanes store one row's 256 contiguous bytes.  A wavefront's LDS accesses execute in
        // order, and the area is its own: no barrier.
        const uint32_t ebase = xs_base + (uint32_t)wave * kEpiWaveBytes;
        const long jbase = ((long)nblock * kGmWaves + wave) * 64;
        const int rsub = lane >> 4, chunk = lane & 15;
        const bool col_ok = strip_ok[chunk >> 3];
        const uint32_t wr = ebase + (uint32_t)ln * kEpiRowBytes + (uint32_t)kb * 16u;
#pragma unroll
        for (int tf = 0; tf < NTF; tf++) {
            const int trow = 32 * tf + ln;
            const int pair_w = (trow < rows) ? perm[row0 + trow] : -1;
#pragma unroll
            for (int s = 0; s < 2; s++)
#pragma unroll
                for (int g = 0; g < 4; g++) {
                    uint4 o;
                    o.x = __float_as_uint(acc[s][tf][4 * g + 0]);
                    o.y = __float_as_uint(acc[s][tf][4 * g + 1]);
                    o.z = __float_as_uint(acc[s][tf][4 * g + 2]);
                    o.w = __float_as_uint(acc[s][tf][4 * g + 3]);
                    lds_write16(wr + (uint32_t)(s * 128 + g * 32), o);
                }
            if (kb == 0) lds_write4(ebase + (uint32_t)ln * kEpiRowBytes + 256u, (uint32_t)pair_w);
#pragma unroll
            for (int j = 0; j < 8; j++) {
                const uint32_t ra = ebase + (uint32_t)(rsub + 4 * j) * kEpiRowBytes;
                const int pair = (int)lds_read4(ra + 256u);
                const uint4 v = lds_read16(ra + (uint32_t)chunk * 16u);
                if (pair >= 0 && col_ok)
                    *reinterpret_cast<uint4*>(oout + (long)pair * N + jbase + 4 * chunk) = v;
            }
        }
        return;
    }
#pragma unroll
    for (int tf = 0; tf < NTF; tf++) {
        const int trow = 32 * tf + ln;
        if (MODE == 1) {
            // SwiGLU; the 16-bit intermediate is written in the column order the
            // down projection of this expert reads (see perm8 / perm16)
            // The workgroup's four strips are 128 adjacent features: every wavefront writes its 64 bytes of each
            // row into LDS (272 bytes per row), and after one barrier the rows go out whole, 16 lanes per row.
            const uint32_t dst = xs_base + (uint32_t)trow * kEpiRowBytes + (uint32_t)wave * 64u;
            uint32_t pk[4][2];
#pragma unroll
            for (int g = 0; g < 4; g++) {
                float hv[4];
#pragma unroll
                for (int i = 0; i < 4; i++) {
                    const float a = acc[0][tf][4 * g + i];
                    const float u = acc[1][tf][4 * g + i];
                    hv[i] = a * __builtin_amdgcn_rcpf(1.0f + __expf(-a)) * u;
                }
                if constexpr (BITS == 16) {
                    pk[g][0] = f32_to_bf16_bits(hv[0]) | (f32_to_bf16_bits(hv[1]) << 16);
                    pk[g][1] = f32_to_bf16_bits(hv[2]) | (f32_to_bf16_bits(hv[3]) << 16);
                } else {
                    pk[g][0] = pack_half2(hv[0], hv[1]);
                    pk[g][1] = pack_half2(hv[2], hv[3]);
                }
            }
            if constexpr (BITS == 16 || BITS == 8) {
                // features f0 + 8g + 4kb .. +4, natural order
#pragma unroll
                for (int g = 0; g < 4; g++) lds_write8(dst + (uint32_t)(2 * (8 * g + 4 * kb)), make_uint2(pk[g][0], pk[g][1]));
            } else if constexpr (BITS == 4) {
                // group of 8 features e0..e7: this lane holds e(4kb..4kb+3); stored order is
                // e0,e4,e1,e5 | e2,e6,e3,e7: the two kb lanes trade one packed pair
#pragma unroll
                for (int g = 0; g < 4; g++) {
                    const uint32_t send = kb ? pk[g][0] : pk[g][1];          // kb0 gives (e2,e3), kb1 gives (e4,e5)
                    const uint32_t got = (uint32_t)__shfl_xor((int)send, 32, kWave);
                    const uint32_t lo = kb ? got : pk[g][0];                 // kb0: (e0,e1)  kb1: (e2,e3)
                    const uint32_t hi = kb ? pk[g][1] : got;                 // kb0: (e4,e5)  kb1: (e6,e7)
                    const uint32_t o0 = (lo & 0xffffu) | (hi << 16);
                    const uint32_t o1 = (lo >> 16) | (hi & 0xffff0000u);
                    lds_write8(dst + (uint32_t)(2 * (8 * g + 4 * kb)), make_uint2(o0, o1));
                }
            } else {
                // group of 16 features = register groups (g, g+1), g even: this lane holds
                // e(4kb+i) and e(8+4kb+i); stored order interleaves them at 8kb .. 8kb+7
                {
#pragma unroll
                    for (int g = 0; g < 4; g += 2) {
                        const uint32_t a01 = pk[g][0], a23 = pk[g][1], b01 = pk[g + 1][0], b23 = pk[g + 1][1];
                        uint4 o;
                        o.x = (a01 & 0xffffu) | (b01 << 16);
                        o.y = (a01 >> 16) | (b01 & 0xffff0000u);
                        o.z = (a23 & 0xffffu) | (b23 << 16);
                        o.w = (a23 >> 16) | (b23 & 0xffff0000u);
                        lds_write16(dst + (uint32_t)(2 * (8 * g + 8 * kb)), o);
                    }
                }
            }
        }
    }
    if (MODE == 1) {
        __syncthreads();
        const long f0 = (long)nblock * (32 * kGmWaves);
        const int chunk = tid & 15;                        // 8 features
        const bool col_ok = f0 + 8 * chunk < N;
        for (int r = tid >> 4; r < rows; r += kGmThreads / 16) {
            const uint4 v = lds_read16(xs_base + (uint32_t)r * kEpiRowBytes + (uint32_t)chunk * 16u);
            if (col_ok) *reinterpret_cast<uint4*>(hout + (long)(row0 + r) * N + f0 + 8 * chunk) = v;
        }
    }
}

template <int MODE>
__global__ __launch_bounds__(kGmThreads, 2) void gemm_kernel(
    const uint16_t* __restrict__ x_bf16, const uint16_t* __restrict__ x_h4,
    const uint16_t* __restrict__ x_h2, const uint16_t* __restrict__ x_h8,
    const uint16_t* __restrict__ hbuf_in,
    const uint8_t* __restrict__ bits, const dymoe_expert_fmt* __restrict__ table,
    const int32_t* __restrict__ plan, int P, int E, int k_route, int H, int F,
    uint16_t* __restrict__ hbuf_out, float* __restrict__ opair, int max_tiles, int splits)
{
    // two token-tile buffers; the swizzle works on the address bits inside a row
    extern __shared__ __attribute__((aligned(1024))) uint16_t xs_raw[];
    const uint32_t xs = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) uint16_t*)xs_raw;
    const PlanPtrs pp = plan_ptrs(const_cast<int32_t*>(plan), E, P);
    const int K = (MODE == 1) ? H : F;
    const int N = (MODE == 1) ? F : H;
    // Which (column block, tile, K split) this workgroup takes.  Both launches are one-dimensional: workgroups go to the
    // 8 XCDs (each with an L2 of its own) in turn by launch index, L -> XCD c = L % 8, place j = L / 8 in that XCD's
    // sequence, and the units (a tile's rows over one K split) are handed out 8 at a time, all their column blocks,
    // before the next 8 (so the longest-first order of the tile list survives).  Inside such a group of 8 units x nblk
    // column blocks one of two things can be shared through an XCD's L2, and the plan says which pays:
    //  * the token rows (second GEMM): the column blocks of a unit all read the same rows of the intermediate.  XCD c
    //    takes unit c of the group in every column block.  Right when an expert has one tile, as in the Mixtral prefill
    //    (the second GEMM read 1.9 x its operands before);
    //  * the weights: tiles of ONE expert are neighbours in the list (equal cost keys keep the expert order) and read the
    //    same weight strips column block by column block.  The group's 8 x nblk (unit, column block) pairs are numbered
    //    column block first, q = 8 * column block + unit, and XCD c takes q in [c * nblk, (c + 1) * nblk): a column
    //    block's strips are then read by at most two XCDs instead of eight.  Right when experts have many tiles (routing
    //    with a few popular experts: the first GEMM of the 128-expert layer streamed 3.4 x its weights, at 5.9 TB/s).
    // The plan counts tiles and experts with tiles; weights are shared when there are at least twice as many tiles.
    int tile, bx, bz;
    {
        const int cols = (MODE == 1) ? 32 * kGmWaves : 64 * kGmWaves;
        const int nblk = (N + cols - 1) / cols;
        const int L = blockIdx.x, c = L & 7, j = L >> 3;
        const int g = j / nblk, sq = j - g * nblk;
        const bool share_weights = pp.ntiles[0] >= 2 * pp.ntiles[2];
        int unit;
        if (share_weights) {
            const int q = c * nblk + sq;
            bx = q >> 3;
            unit = 8 * g + (q & 7);
        } else if (MODE == 2) {
            bx = sq;
            unit = 8 * g + c;
        } else {
            // (first GEMM, one tile per expert: a tile per XCD would give each XCD one format, and the formats differ in
            // cost per tile; the tile's column blocks go round all XCDs instead, launch index = tile * nblk + column block)
            unit = L / nblk;
            bx = L - unit * nblk;
        }
        tile = unit / splits;
        bz = unit - tile * splits;
        if (tile >= max_tiles) return;
    }
    if (tile >= pp.ntiles[0]) return;
    const int e = pp.tiles[4 * tile + 0];
    const int row0 = pp.tiles[4 * tile + 1];
    const int rows = pp.tiles[4 * tile + 2];
    const int b = bits[e];
    const dymoe_expert_fmt ex = table[e];
    // split-K (second GEMM only): split bz takes K-tiles [bz*per, (bz+1)*per) and its own output slab
    const int nkt = K / kBK;
    const int per = (nkt + splits - 1) / splits;
    const int kt_begin = bz * per;
    const int kt_end = min(nkt, kt_begin + per);
    float* oz = opair + (size_t)bz * (size_t)P * (size_t)N;
    if (kt_begin >= kt_end) {
        // a split with no K-tiles still owns its slab: write zeros
        if (MODE == 2) {
            const int cols = 64 * kGmWaves;     // columns of this workgroup
            for (int i = threadIdx.x; i < rows * (cols / 4); i += kGmThreads) {
                const int r = i / (cols / 4), c = bx * cols + (i % (cols / 4)) * 4;
                if (c < N)
                    *reinterpret_cast<float4*>(oz + (size_t)pp.perm[row0 + r] * N + c) = make_float4(0.f, 0.f, 0.f, 0.f);
            }
        }
        return;
    }
    const uint16_t* act = (MODE != 1) ? hbuf_in : (b == 16 ? x_bf16 : (b == 8 ? x_h8 : (b == 4 ? x_h4 : x_h2)));
    const int ntf = (rows + 31) >> 5;
    // one instantiation per (precision, number of 32-token fragments): the
    // accumulators then sit in fixed registers for the whole K loop
#define DYMOE_TILE(BITS_, NTF_)                                                                      \
    gemm_tile<MODE, BITS_, NTF_>(act, pp.perm, k_route, ex, K, N, kt_begin, kt_end, row0, rows,      \
                                 bx, hbuf_out, oz, xs)
#define DYMOE_TILE_NTF(BITS_)                     \
    switch (ntf) {                                \
    case 1: DYMOE_TILE(BITS_, 1); break;          \
    case 2: DYMOE_TILE(BITS_, 2); break;          \
    case 3: DYMOE_TILE(BITS_, 3); break;          \
    case 4: DYMOE_TILE(BITS_, 4); break;          \
    default:                                      \
        if constexpr (BITS_ == 4 || BITS_ == 2) { \
            DYMOE_TILE(BITS_, 5);                 \
        } else {                                  \
            DYMOE_TILE(BITS_, 4);                 \
        }                                         \
        break;                                    \
    }
    if (b == 16) {
        DYMOE_TILE_NTF(16)
    } else if (b == 8) {
        DYMOE_TILE_NTF(8)
    } else if (b == 4) {
        DYMOE_TILE_NTF(4)
    } else {
        DYMOE_TILE_NTF(2)
    }
#undef DYMOE_TILE_NTF
#undef DYMOE_TILE
}

// y[t,j] = sum_slot w[t,slot] * (sum over K splits of o[z,pair,j])  (pairs of skipped experts omitted)
__global__ __launch_bounds__(256) void gemm_combine_kernel(
    const float* __restrict__ opair, const int32_t* __restrict__ idx, const float* __restrict__ w,
    const uint8_t* __restrict__ bits, int T, int H, int E, int k, int splits, int out_dtype,
    void* __restrict__ y)
{
    const long i4 = (long)blockIdx.x * 256 + threadIdx.x;  // groups of 4 columns
    const long n4 = (long)T * (H >> 2);
    if (i4 >= n4) return;
    const int t = (int)(i4 / (H >> 2));
    const int j = (int)(i4 - (long)t * (H >> 2)) * 4;
    float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
    for (int slot = 0; slot < k; slot++) {
        const int p = t * k + slot;
        const int e = idx[p];
        if (e < 0 || e >= E) continue;
        const int b = bits[e];
        if (b != 16 && b != 8 && b != 4 && b != 2) continue;
        const float g = w[p];
        float4 o = *reinterpret_cast<const float4*>(opair + (long)p * H + j);
        for (int z = 1; z < splits; z++) {
            const float4 oz = *reinterpret_cast<const float4*>(opair + ((long)z * T * k + p) * H + j);
            o.x += oz.x; o.y += oz.y; o.z += oz.z; o.w += oz.w;
        }
        acc.x = fmaf(g, o.x, acc.x);
        acc.y = fmaf(g, o.y, acc.y);
        acc.z = fmaf(g, o.z, acc.z);
        acc.w = fmaf(g, o.w, acc.w);
    }
    if (out_dtype == DYMOE_OUT_F32) {
        *reinterpret_cast<float4*>(reinterpret_cast<float*>(y) + (long)t * H + j) = acc;
    } else {
        uint2 pk;
        pk.x = f32_to_bf16_bits(acc.x) | (f32_to_bf16_bits(acc.y) << 16);
        pk.y = f32_to_bf16_bits(acc.z) | (f32_to_bf16_bits(acc.w) << 16);
        *reinterpret_cast<uint2*>(reinterpret_cast<uint16_t*>(y) + (long)t * H + j) = pk;
    }
}

constexpr size_t kGemmLdsBytes = 2 * (size_t)kXsBufBytes;     // two token-tile buffers

// Once per device, at context creation, with that device current: the kernels use more dynamic LDS than the default limit.
int ffn_gemm_init()
{
    if (hipFuncSetAttribute(reinterpret_cast<const void*>(&gemm_kernel<1>),
                            hipFuncAttributeMaxDynamicSharedMemorySize, (int)kGemmLdsBytes) != hipSuccess ||
        hipFuncSetAttribute(reinterpret_cast<const void*>(&gemm_kernel<2>),
                            hipFuncAttributeMaxDynamicSharedMemorySize, (int)kGemmLdsBytes) != hipSuccess)
        return DYMOE_EHIP;
    return DYMOE_OK;
}

// Limits of the launch shapes below, checked by the entry point before anything is enqueued: the tile index is a
// grid's y dimension, and the token-tile copies address a row through an unsigned 32-bit byte offset.
bool ffn_gemm_fits(int T, int H, int F, int E, int k)
{
    const size_t P = (size_t)T * (size_t)k;
    const size_t tiles = P / kGemmTileM + (size_t)E;
    if (tiles > 65535) return false;
    // both launches are one-dimensional: 8 * column blocks * ceil(units / 8) workgroups, units <= 8 * tiles
    const size_t nblk = ((size_t)(F > H ? F : H) + 32 * kGmWaves - 1) / (32 * kGmWaves);
    if (8 * nblk * (tiles + 1) >= ((size_t)1 << 31)) return false;
    if ((size_t)T * H * 2 >= ((size_t)1 << 32) || P * (size_t)F * 2 >= ((size_t)1 << 32)) return false;
    return true;
}

int ffn_gemm_launch(dymoe_ctx* ctx, const void* x, const int32_t* idx, const float* w, const uint8_t* bits,
                    const dymoe_expert_fmt* table, int T, int H, int F, int E, int k,
                    int out_dtype, void* y, void* workspace, hipStream_t st)
{
    const FfnLayout L = ffn_layout(T, H, F, E, k);
    const int P = T * k;
    if (!ffn_gemm_fits(T, H, F, E, k)) return DYMOE_ENOTSUP;
    char* ws = (char*)workspace;
    uint16_t* hbuf = reinterpret_cast<uint16_t*>(ws + L.hbuf);   // [P,F] 16-bit
    uint16_t* xh4 = reinterpret_cast<uint16_t*>(ws + L.xh);      // [T,H] fp16, int4 column order
    uint16_t* xh2 = xh4 + round256((size_t)T * H * 2) / 2;       // [T,H] fp16, int2 column order
    uint16_t* xh8 = xh2 + round256((size_t)T * H * 2) / 2;       // [T,H] fp16, natural column order (int8)
    float* opair = reinterpret_cast<float*>(ws + L.part);
    int32_t* plan = reinterpret_cast<int32_t*>(ws + L.plan);
    const uint16_t* xb = (const uint16_t*)x;

    dymoe_launch(ctx, DYMOE_K_PLAN, plan_kernel, dim3(1), dim3(kPlanThreads), 0, st, idx, bits, table, P, E, kGemmTileM,
                 L.max_tiles, plan, ctx->device_flags);
    // what the kernels after the plan take as the bit widths: the plan's copy, 0 where the table lacks the format
    const uint8_t* run_bits = reinterpret_cast<const uint8_t*>(plan_ptrs(plan, E, P).cursor);
    DYMOE_HIP_LAUNCH_CHECK();
    const long n16 = (long)T * H / 16;
    hipLaunchKernelGGL(prep_x_kernel, dim3((unsigned)((n16 + 255) / 256)), dim3(256), 0, st, xb, n16, xh4, xh2, xh8);
    DYMOE_HIP_LAUNCH_CHECK();
    constexpr size_t kLdsBytes = kGemmLdsBytes;
    const int max_tiles = P / kGemmTileM + E;
    const int cols1 = 32 * kGmWaves, cols2 = 64 * kGmWaves;
    const int nblk1 = (F + cols1 - 1) / cols1;
    const dim3 g1((unsigned)(8 * nblk1 * ((max_tiles + 7) / 8)));
    dymoe_launch(ctx, DYMOE_K_GEMM1, (gemm_kernel<1>), g1, dim3(kGmThreads), kLdsBytes, st, xb, xh4, xh2, xh8,
                 (const uint16_t*)nullptr, run_bits, table, plan, P, E, k, H, F, hbuf, (float*)nullptr, max_tiles, 1);
    DYMOE_HIP_LAUNCH_CHECK();
    // The down projection has few output tiles: split K so that the launch still covers the chip (two workgroups per
    // compute unit, about one and a half rounds of them; measured on the Mixtral prefill: 2 to 7 splits lie within
    // 7 % of each other, 4 is best).  Each split writes its own slab of per-pair outputs and the combine kernel adds
    // the slabs in a fixed order, so every extra split also costs a slab of traffic each way.  The number of tiles is
    // only known on the device; from the sizes: every expert with tokens has one, and P / 128 more at most.
    const int nblk2 = (H + cols2 - 1) / cols2;
    const long est_tiles = (E < P ? E : P) + (long)P / (2 * kGemmTileM);
    const long est_blocks = (long)nblk2 * est_tiles;
    int splits = (int)(3L * ctx->num_cu / est_blocks);
    const int max_splits = (F + kSeg - 1) / kSeg;     // slabs the workspace holds
    if (splits > max_splits) splits = max_splits;
    if (splits > 8) splits = 8;
    if (splits < 1) splits = 1;
    const int units = max_tiles * splits;
    const dim3 g2((unsigned)(8 * nblk2 * ((units + 7) / 8)));
    dymoe_launch(ctx, DYMOE_K_GEMM2, (gemm_kernel<2>), g2, dim3(kGmThreads), kLdsBytes, st, xb, xh4, xh2, xh8, hbuf,
                 run_bits, table, plan, P, E, k, H, F, (uint16_t*)nullptr, opair, max_tiles, splits);
    DYMOE_HIP_LAUNCH_CHECK();
    const long n4 = (long)T * (H / 4);
    dymoe_launch(ctx, DYMOE_K_GEMM_COMBINE, gemm_combine_kernel, dim3((unsigned)((n4 + 255) / 256)), dim3(256), 0, st, opair,
                 idx, w, run_bits, T, H, E, k, splits, out_dtype, y);
    DYMOE_HIP_LAUNCH_CHECK();
    return DYMOE_OK;
}

}  // namespace dymoe
