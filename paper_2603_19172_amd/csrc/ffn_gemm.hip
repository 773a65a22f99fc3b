// Prefill path of the mixed-precision SwiGLU expert FFN: tokens grouped by
// expert, one MFMA grouped GEMM per projection, all experts in one launch.
//
// Tile: up to 128 token rows of one expert x (4 wavefronts x 2 strips of 32
// weight rows), K-blocks of 128.  Weights never touch LDS: the MFMA A operand
// of lane (r, kb) is 8 consecutive k of weight row r, so every lane loads its
// own row's bytes straight from HBM (bf16: as is; int4 / int2: packed codes,
// turned into fp16 in registers).  The contraction order inside a K-block is
// permuted so that one lane's 64 k (one quantisation group) are contiguous in
// memory; the token tile in LDS is stored in the matching order.
//   bf16 experts: v_mfma_f32_32x32x16_bf16 on the bf16 activations
//   int4 / int2 : v_mfma_f32_32x32x16_f16 on an fp16 copy of the activations,
//                 weights dequantised as fma(q, s, m) in packed fp16
// Code fields become fp16 numbers by OR-ing them into the mantissa of 2^n
// (n such that the field's lowest bit weighs one), then subtracting 2^n.
#include <math.h>

#include "common.hpp"
#include "ffn_layout.hpp"

namespace dymoe {

constexpr int kGmThreads = 256;
constexpr int kGmWaves = 4;
constexpr int kBK = 128;            // K-block
constexpr int kLdsStride = 136;     // 16-bit elements per LDS row (128 + pad, keeps b128 reads conflict free)

// ----------------------------------------------------------------------------
// plan: counting sort of the (token, slot) pairs by expert + tile list
// ints: counts[E] | offsets[E+1] | cursor[E] | ntiles (8 ints) | perm[P] | tiles[4*max_tiles]
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

__global__ __launch_bounds__(1024) void plan_kernel(const int32_t* __restrict__ idx,
                                                    const uint8_t* __restrict__ bits, int P, int E,
                                                    int tile_m, int32_t* __restrict__ plan)
{
    __shared__ int32_t s_count[DYMOE_MAX_EXPERTS];
    __shared__ int32_t s_off[DYMOE_MAX_EXPERTS + 1];
    const PlanPtrs pp = plan_ptrs(plan, E, P);
    for (int e = threadIdx.x; e < E; e += blockDim.x) s_count[e] = 0;
    __syncthreads();
    for (int p = threadIdx.x; p < P; p += blockDim.x) {
        const int e = idx[p];
        if (e < 0 || e >= E) continue;
        const int b = bits[e];
        if (b != 16 && b != 4 && b != 2) continue;
        atomicAdd(&s_count[e], 1);
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        int run = 0, nt = 0;
        for (int e = 0; e < E; e++) {
            s_off[e] = run;
            const int c = s_count[e];
            for (int m0 = 0; m0 < c; m0 += tile_m) {
                pp.tiles[4 * nt + 0] = e;
                pp.tiles[4 * nt + 1] = run + m0;
                pp.tiles[4 * nt + 2] = min(tile_m, c - m0);
                pp.tiles[4 * nt + 3] = 0;
                nt++;
            }
            run += c;
        }
        s_off[E] = run;
        pp.ntiles[0] = nt;
        pp.ntiles[1] = run;
    }
    __syncthreads();
    for (int e = threadIdx.x; e < E; e += blockDim.x) {
        pp.counts[e] = s_count[e];
        pp.offsets[e] = s_off[e];
        s_count[e] = 0;  // reused as the scatter cursor
    }
    if (threadIdx.x == 0) pp.offsets[E] = s_off[E];
    __syncthreads();
    // order inside an expert is arbitrary: every row of a tile is computed independently
    for (int p = threadIdx.x; p < P; p += blockDim.x) {
        const int e = idx[p];
        if (e < 0 || e >= E) continue;
        const int b = bits[e];
        if (b != 16 && b != 4 && b != 2) continue;
        const int pos = s_off[e] + atomicAdd(&s_count[e], 1);
        pp.perm[pos] = p;
    }
}

// fp16 copy of the bf16 activations (exact inside fp16's normal range)
__global__ __launch_bounds__(256) void to_f16_kernel(const uint16_t* __restrict__ x, long n8,
                                                     uint16_t* __restrict__ out)
{
    const long i = (long)blockIdx.x * 256 + threadIdx.x;
    if (i >= n8) return;
    const uint4 v = reinterpret_cast<const uint4*>(x)[i];
    uint4 o;
    o.x = pack_half2(bf16_lo(v.x), bf16_hi(v.x));
    o.y = pack_half2(bf16_lo(v.y), bf16_hi(v.y));
    o.z = pack_half2(bf16_lo(v.z), bf16_hi(v.z));
    o.w = pack_half2(bf16_lo(v.w), bf16_hi(v.w));
    reinterpret_cast<uint4*>(out)[i] = o;
}

// ----------------------------------------------------------------------------
// weight strips

template <int BITS> struct StripRaw;
template <> struct StripRaw<16> { uint4 r[8]; };
template <> struct StripRaw<4> { uint4 r[2]; uint32_t s2, m2; };
template <> struct StripRaw<2> { uint4 r[1]; uint32_t s2, m2; };

struct MatPtr {
    const uint16_t* w;
    const uint8_t* q;
    const uint16_t* s;
    const uint16_t* z;
};

__device__ __forceinline__ MatPtr mat_ptr(const dymoe_expert_fmt& ex, int mat, int b)
{
    MatPtr m;
    m.w = reinterpret_cast<const uint16_t*>(ex.w[mat]);
    m.q = (b == 4) ? ex.q4[mat] : ex.q2[mat];
    m.s = reinterpret_cast<const uint16_t*>((b == 4) ? ex.s4[mat] : ex.s2[mat]);
    m.z = reinterpret_cast<const uint16_t*>((b == 4) ? ex.z4[mat] : ex.z2[mat]);
    return m;
}

// lane (n, kb) of a strip loads k in [k0 + 64 kb, k0 + 64 kb + 64) of weight row n
template <int BITS>
__device__ __forceinline__ void load_strip(const MatPtr& m, long n, int kb, int k0, int K,
                                           StripRaw<BITS>& raw)
{
    const int kk = k0 + 64 * kb;
    if constexpr (BITS == 16) {
        const uint4* src = reinterpret_cast<const uint4*>(m.w + n * K + kk);
#pragma unroll
        for (int j = 0; j < 8; j++) raw.r[j] = src[j];
    } else if constexpr (BITS == 4) {
        const uint4* src = reinterpret_cast<const uint4*>(m.q + n * (long)(K >> 1) + (kk >> 1));
        StripRaw<4>& r4 = raw;
        r4.r[0] = src[0];
        r4.r[1] = src[1];
        const long g = n * (long)(K >> 6) + (kk >> 6);
        const uint32_t s = m.s[g], z = m.z[g];
        r4.s2 = s | (s << 16);
        r4.m2 = z | (z << 16);
    } else {
        const uint4* src = reinterpret_cast<const uint4*>(m.q + n * (long)(K >> 2) + (kk >> 2));
        StripRaw<2>& r2 = raw;
        r2.r[0] = src[0];
        const long g = n * (long)(K >> 6) + (kk >> 6);
        const uint32_t s = m.s[g], z = m.z[g];
        r2.s2 = s | (s << 16);
        r2.m2 = z | (z << 16);
    }
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
    } else if constexpr (BITS == 4) {
        const StripRaw<4>& r = raw;
        const uint4 q = r.r[jj >> 1];
        const uint32_t w0 = (jj & 1) ? q.z : q.x;
        const uint32_t w1 = (jj & 1) ? q.w : q.y;
        // k order inside a fragment: 0,4,1,5,2,6,3,7
        uint32_t v = w0, v8 = w0 >> 8;
        f0.x = deq_pair((v & 0x000F000Fu) | 0x64006400u, 0x64006400u, r.s2, r.m2);
        f0.y = deq_pair((v & 0x00F000F0u) | 0x54005400u, 0x54005400u, r.s2, r.m2);
        f0.z = deq_pair((v8 & 0x000F000Fu) | 0x64006400u, 0x64006400u, r.s2, r.m2);
        f0.w = deq_pair((v8 & 0x00F000F0u) | 0x54005400u, 0x54005400u, r.s2, r.m2);
        v = w1; v8 = w1 >> 8;
        f1.x = deq_pair((v & 0x000F000Fu) | 0x64006400u, 0x64006400u, r.s2, r.m2);
        f1.y = deq_pair((v & 0x00F000F0u) | 0x54005400u, 0x54005400u, r.s2, r.m2);
        f1.z = deq_pair((v8 & 0x000F000Fu) | 0x64006400u, 0x64006400u, r.s2, r.m2);
        f1.w = deq_pair((v8 & 0x00F000F0u) | 0x54005400u, 0x54005400u, r.s2, r.m2);
    } else {
        const StripRaw<2>& r = raw;
        const uint4 q = r.r[0];
        const uint32_t v = (jj == 0) ? q.x : (jj == 1) ? q.y : (jj == 2) ? q.z : q.w;
        const uint32_t v10 = v >> 10;
        // 16 codes of the dword; k order 0,8,1,9,2,10,3,11 | 4,12,5,13,6,14,7,15
        f0.x = deq_pair((v & 0x00030003u) | 0x64006400u, 0x64006400u, r.s2, r.m2);
        f0.y = deq_pair((v & 0x000C000Cu) | 0x5C005C00u, 0x5C005C00u, r.s2, r.m2);
        f0.z = deq_pair((v & 0x00300030u) | 0x54005400u, 0x54005400u, r.s2, r.m2);
        f0.w = deq_pair((v & 0x00C000C0u) | 0x4C004C00u, 0x4C004C00u, r.s2, r.m2);
        f1.x = deq_pair((v & 0x03000300u) | 0x44004400u, 0x44004400u, r.s2, r.m2);
        f1.y = deq_pair((v10 & 0x00030003u) | 0x64006400u, 0x64006400u, r.s2, r.m2);
        f1.z = deq_pair((v10 & 0x000C000Cu) | 0x5C005C00u, 0x5C005C00u, r.s2, r.m2);
        f1.w = deq_pair((v10 & 0x00300030u) | 0x54005400u, 0x54005400u, r.s2, r.m2);
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

// reorder 8 (int4) or 16 (int2) consecutive 16-bit activations into the k
// order in which the code fields come out of a dword
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

// one K-block of MFMAs for NTF token fragments (32 tokens each)
template <int BITS, int NTF>
__device__ __forceinline__ void compute_kblock(const StripRaw<BITS>& ra, const StripRaw<BITS>& rb,
                                               const uint16_t (*xs)[kLdsStride], int ln, int kb,
                                               float16_t (&acc)[2][NTF])
{
#pragma unroll
    for (int jj = 0; jj < 4; jj++) {
        uint4 a0, a1, b0, b1;
        strip_frags<BITS>(ra, jj, a0, a1);
        strip_frags<BITS>(rb, jj, b0, b1);
#pragma unroll
        for (int tf = 0; tf < NTF; tf++) {
            const uint4 t0 = *reinterpret_cast<const uint4*>(&xs[32 * tf + ln][64 * kb + 16 * jj]);
            const uint4 t1 = *reinterpret_cast<const uint4*>(&xs[32 * tf + ln][64 * kb + 16 * jj + 8]);
            acc[0][tf] = mfma16<BITS>(a0, t0, acc[0][tf]);
            acc[1][tf] = mfma16<BITS>(b0, t0, acc[1][tf]);
            acc[0][tf] = mfma16<BITS>(a1, t1, acc[0][tf]);
            acc[1][tf] = mfma16<BITS>(b1, t1, acc[1][tf]);
        }
    }
}

// ----------------------------------------------------------------------------
// MODE 1: h = silu(x W1^T) * (x W3^T)   strips = (W1 rows, W3 rows) of the same 32 features
// MODE 2: o = h W2^T                     strips = two adjacent groups of 32 rows of W2,
//                                        K range [k_begin, k_end) of the split
// The K loop is software pipelined: while K-block i is multiplied out of
// registers (weights) and LDS buffer i&1 (tokens), the weights of K-block i+1
// are in flight to registers and its token tile is in flight to registers, to
// be written to the other LDS buffer afterwards; one barrier per K-block.
template <int MODE, int BITS, int NTF>
__device__ __forceinline__ void gemm_tile(
    const uint16_t* __restrict__ act,   // MODE 1: [T,H] activations (gathered); MODE 2: [P,F] intermediate
    const int32_t* __restrict__ perm, int k_route, const dymoe_expert_fmt& ex, int K, int N,
    int k_begin, int k_end, int row0, int rows, int nblock, uint16_t* __restrict__ hout,
    float* __restrict__ oout, uint16_t (*xs)[kGemmTileM][kLdsStride])
{
    const int tid = threadIdx.x;
    const int lane = tid & (kWave - 1);
    const int wave = tid / kWave;
    const int ln = lane & 31;
    const int kb = lane >> 5;

    // strips of this wavefront
    long n_a, n_b;
    MatPtr ma, mb;
    bool strip_ok[2];
    if (MODE == 1) {
        const int f0 = nblock * (32 * kGmWaves) + wave * 32;
        n_a = n_b = f0 + ln;
        ma = mat_ptr(ex, 0, BITS);
        mb = mat_ptr(ex, 1, BITS);
        strip_ok[0] = strip_ok[1] = f0 < N;
    } else {
        const int j0 = nblock * (64 * kGmWaves) + wave * 64;
        n_a = j0 + ln;
        n_b = j0 + 32 + ln;
        ma = mb = mat_ptr(ex, 2, BITS);
        strip_ok[0] = j0 < N;
        strip_ok[1] = j0 + 32 < N;
    }
    if (!strip_ok[0]) n_a = 0;
    if (!strip_ok[1]) n_b = 0;

    float16_t acc[2][NTF];
#pragma unroll
    for (int s = 0; s < 2; s++)
#pragma unroll
        for (int tf = 0; tf < NTF; tf++)
#pragma unroll
            for (int i = 0; i < 16; i++) acc[s][tf][i] = 0.0f;

    // staging role: thread -> (row, half) of the token tile
    const int srow = tid >> 1;
    const int shalf = tid & 1;
    // tile rows past the expert's last token re-read its last token: their
    // products are computed and dropped, and the loop stays branch-free
    const int srow_c = min(srow, rows - 1);
    const uint16_t* src_row;
    if (MODE == 1) src_row = act + (long)(perm[row0 + srow_c] / k_route) * K;
    else src_row = act + (long)(row0 + srow_c) * K;
    uint4 xv[8];
    auto load_x = [&](int k0) {
#pragma unroll
        for (int i = 0; i < 8; i++)
            xv[i] = *reinterpret_cast<const uint4*>(src_row + k0 + 64 * shalf + 8 * i);
    };
    auto store_x = [&](int buf) {
        uint4* dst = reinterpret_cast<uint4*>(&xs[buf][srow][64 * shalf]);
        if constexpr (BITS == 16) {
#pragma unroll
            for (int i = 0; i < 8; i++) dst[i] = xv[i];
        } else if constexpr (BITS == 4) {
#pragma unroll
            for (int i = 0; i < 8; i++) dst[i] = perm8(xv[i]);
        } else {
#pragma unroll
            for (int i = 0; i < 4; i++) {
                uint4 o0, o1;
                perm16(xv[2 * i], xv[2 * i + 1], o0, o1);
                dst[2 * i] = o0;
                dst[2 * i + 1] = o1;
            }
        }
    };

    // Two register sets (0 / 1) take turns, so no value is ever copied from a
    // "next" to a "current" register: a copy would have to wait for the loads
    // it copies.  The scheduler fences keep the prefetch loads at the top of
    // each half-step, ahead of the MFMA work that hides their latency.
    StripRaw<BITS> ra0, rb0, ra1, rb1;
    load_x(k_begin);
    load_strip<BITS>(ma, n_a, kb, k_begin, K, ra0);
    load_strip<BITS>(mb, n_b, kb, k_begin, K, rb0);
    store_x(0);
    __syncthreads();
    for (int k0 = k_begin; k0 < k_end; k0 += 2 * kBK) {
        // half-step A: prefetch block k0 + BK into set 1, multiply set 0 from LDS buffer 0
        // (past the end the prefetch re-reads the last block instead of branching)
        const int k1 = min(k0 + kBK, k_end - kBK);
        load_x(k1);
        load_strip<BITS>(ma, n_a, kb, k1, K, ra1);
        load_strip<BITS>(mb, n_b, kb, k1, K, rb1);
        __builtin_amdgcn_sched_barrier(0);
        compute_kblock<BITS, NTF>(ra0, rb0, xs[0], ln, kb, acc);
        __builtin_amdgcn_sched_barrier(0);
        store_x(1);
        __syncthreads();
        if (k0 + kBK >= k_end) break;   // odd number of K-blocks
        // half-step B: prefetch block k0 + 2 BK into set 0, multiply set 1 from LDS buffer 1
        const int k2 = min(k0 + 2 * kBK, k_end - kBK);
        load_x(k2);
        load_strip<BITS>(ma, n_a, kb, k2, K, ra0);
        load_strip<BITS>(mb, n_b, kb, k2, K, rb0);
        __builtin_amdgcn_sched_barrier(0);
        compute_kblock<BITS, NTF>(ra1, rb1, xs[1], ln, kb, acc);
        __builtin_amdgcn_sched_barrier(0);
        store_x(0);
        __syncthreads();
    }

    // epilogue.  D layout: lane (ln, kb), register i -> weight row 8*(i/4) + 4*kb + i%4, token ln
#pragma unroll
    for (int tf = 0; tf < NTF; tf++) {
        const int trow = 32 * tf + ln;
        if (trow < rows) {
            if (MODE == 1) {
                if (strip_ok[0]) {
                    const int f0 = nblock * (32 * kGmWaves) + wave * 32;
                    uint16_t* dst = hout + (long)(row0 + trow) * N + f0 + 4 * kb;
#pragma unroll
                    for (int g = 0; g < 4; g++) {
                        float hv[4];
#pragma unroll
                        for (int i = 0; i < 4; i++) {
                            const float a = acc[0][tf][4 * g + i];
                            const float u = acc[1][tf][4 * g + i];
                            hv[i] = a * __builtin_amdgcn_rcpf(1.0f + __expf(-a)) * u;
                        }
                        uint2 pk;
                        if (BITS == 16) {
                            pk.x = f32_to_bf16_bits(hv[0]) | (f32_to_bf16_bits(hv[1]) << 16);
                            pk.y = f32_to_bf16_bits(hv[2]) | (f32_to_bf16_bits(hv[3]) << 16);
                        } else {
                            pk.x = pack_half2(hv[0], hv[1]);
                            pk.y = pack_half2(hv[2], hv[3]);
                        }
                        *reinterpret_cast<uint2*>(dst + 8 * g) = pk;
                    }
                }
            } else {
                const int pair = perm[row0 + trow];
#pragma unroll
                for (int s = 0; s < 2; s++) {
                    if (strip_ok[s]) {
                        const int j0 = nblock * (64 * kGmWaves) + wave * 64 + 32 * s;
                        float* dst = oout + (long)pair * N + j0 + 4 * kb;
#pragma unroll
                        for (int g = 0; g < 4; g++) {
                            float4 o;
                            o.x = acc[s][tf][4 * g + 0];
                            o.y = acc[s][tf][4 * g + 1];
                            o.z = acc[s][tf][4 * g + 2];
                            o.w = acc[s][tf][4 * g + 3];
                            *reinterpret_cast<float4*>(dst + 8 * g) = o;
                        }
                    }
                }
            }
        }
    }
}

template <int MODE>
__global__ __launch_bounds__(kGmThreads) void gemm_kernel(
    const uint16_t* __restrict__ x_bf16, const uint16_t* __restrict__ x_f16,
    const uint16_t* __restrict__ hbuf_in, const uint8_t* __restrict__ bits,
    const dymoe_expert_fmt* __restrict__ table, const int32_t* __restrict__ plan, int P, int E,
    int k_route, int H, int F, uint16_t* __restrict__ hbuf_out, float* __restrict__ opair)
{
    extern __shared__ __attribute__((aligned(16))) uint16_t xs_raw[];
    uint16_t (*xs)[kGemmTileM][kLdsStride] = reinterpret_cast<uint16_t (*)[kGemmTileM][kLdsStride]>(xs_raw);
    const PlanPtrs pp = plan_ptrs(const_cast<int32_t*>(plan), E, P);
    const int tile = blockIdx.y;
    if (tile >= pp.ntiles[0]) return;
    const int e = pp.tiles[4 * tile + 0];
    const int row0 = pp.tiles[4 * tile + 1];
    const int rows = pp.tiles[4 * tile + 2];
    const int b = bits[e];
    const dymoe_expert_fmt ex = table[e];
    const int K = (MODE == 1) ? H : F;
    const int N = (MODE == 1) ? F : H;
    // split-K (MODE 2 only): blockIdx.z takes K-blocks [z*per, (z+1)*per) and its own output slab
    const int nkb = K / kBK;
    const int per = (nkb + (int)gridDim.z - 1) / (int)gridDim.z;
    const int k_begin = (int)blockIdx.z * per * kBK;
    const int k_end = min(K, k_begin + per * kBK);
    float* oz = opair + (size_t)blockIdx.z * (size_t)P * (size_t)N;
    if (k_begin >= k_end) {
        // a split with no K-blocks still owns its slab: write zeros
        if (MODE == 2) {
            for (int i = threadIdx.x; i < rows * 64; i += kGmThreads) {
                const int r = i >> 6, c = (blockIdx.x * 64 + (i & 63)) * 4;
                if (c < N) *reinterpret_cast<float4*>(oz + (size_t)pp.perm[row0 + r] * N + c) = make_float4(0.f, 0.f, 0.f, 0.f);
            }
        }
        return;
    }
    const uint16_t* act = (MODE != 1) ? hbuf_in : (b == 16 ? x_bf16 : x_f16);
    const int ntf = (rows + 31) >> 5;
    // one instantiation per (precision, number of 32-token fragments): the
    // accumulators then sit in fixed registers for the whole K loop
#define DYMOE_TILE(BITS_, NTF_)                                                                      \
    gemm_tile<MODE, BITS_, NTF_>(act, pp.perm, k_route, ex, K, N, k_begin, k_end, row0, rows,        \
                                 blockIdx.x, hbuf_out, oz, xs)
#define DYMOE_TILE_NTF(BITS_)                     \
    switch (ntf) {                                \
    case 1: DYMOE_TILE(BITS_, 1); break;          \
    case 2: DYMOE_TILE(BITS_, 2); break;          \
    case 3: DYMOE_TILE(BITS_, 3); break;          \
    default: DYMOE_TILE(BITS_, 4); break;         \
    }
    if (b == 16) {
        DYMOE_TILE_NTF(16)
    } else if (b == 4) {
        DYMOE_TILE_NTF(4)
    } else {
        DYMOE_TILE_NTF(2)
    }
#undef DYMOE_TILE_NTF
#undef DYMOE_TILE
}

// y[t,j] = sum_slot w[t,slot] * o[pair,j]  (pairs of skipped experts omitted)
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
        if (b != 16 && b != 4 && b != 2) continue;
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

int ffn_gemm_launch(dymoe_ctx* ctx, const void* x, const int32_t* idx, const float* w, const uint8_t* bits,
                    const dymoe_expert_fmt* table, int T, int H, int F, int E, int k,
                    int out_dtype, void* y, void* workspace, hipStream_t st)
{
    const FfnLayout L = ffn_layout(T, H, F, E, k);
    const int P = T * k;
    char* ws = (char*)workspace;
    uint16_t* hbuf = reinterpret_cast<uint16_t*>(ws + L.hbuf);   // [P,F] 16-bit
    uint16_t* xh = reinterpret_cast<uint16_t*>(ws + L.xh);       // [T,H] fp16 copy of x
    float* opair = reinterpret_cast<float*>(ws + L.part);
    int32_t* plan = reinterpret_cast<int32_t*>(ws + L.plan);
    const uint16_t* xb = (const uint16_t*)x;

    {
        dymoe_launch(ctx, DYMOE_K_PLAN, plan_kernel, dim3(1), dim3(1024), 0, st, idx, bits, P, E, kGemmTileM, plan);
    }
    DYMOE_HIP_LAUNCH_CHECK();
    const long n8 = (long)T * H / 8;
    hipLaunchKernelGGL(to_f16_kernel, dim3((unsigned)((n8 + 255) / 256)), dim3(256), 0, st, xb, n8, xh);
    DYMOE_HIP_LAUNCH_CHECK();
    // two token-tile buffers in LDS: more than the 64 KiB a kernel gets by default
    constexpr size_t kLdsBytes = 2 * sizeof(uint16_t) * kGemmTileM * kLdsStride;
    static bool lds_attr_set = false;
    if (!lds_attr_set) {
        if (hipFuncSetAttribute(reinterpret_cast<const void*>(&gemm_kernel<1>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, (int)kLdsBytes) != hipSuccess ||
            hipFuncSetAttribute(reinterpret_cast<const void*>(&gemm_kernel<2>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, (int)kLdsBytes) != hipSuccess)
            return DYMOE_EHIP;
        lds_attr_set = true;
    }
    const int max_tiles = P / kGemmTileM + E;
    const dim3 g1((unsigned)((F + 127) / 128), (unsigned)max_tiles);
    dymoe_launch(ctx, DYMOE_K_GEMM1, (gemm_kernel<1>), g1, dim3(kGmThreads), kLdsBytes, st, xb, xh,
                 (const uint16_t*)nullptr, bits, table, plan, P, E, k, H, F, hbuf, (float*)nullptr);
    DYMOE_HIP_LAUNCH_CHECK();
    // The down projection has few output tiles (H/256 per token tile): split K so
    // that the launch still covers the chip.  Each split writes its own slab of
    // per-pair outputs; the combine kernel adds the slabs in a fixed order.
    const int nblk2 = (H + 255) / 256;
    const long est_blocks = (long)nblk2 * ((long)P / kGemmTileM + (E < P ? E : P) / 2 + 1);
    int splits = (int)((2L * ctx->num_cu + est_blocks - 1) / est_blocks);
    const int max_splits = (F + kSeg - 1) / kSeg;     // slabs the workspace holds
    if (splits > max_splits) splits = max_splits;
    if (splits > 4) splits = 4;
    if (splits < 1) splits = 1;
    const dim3 g2((unsigned)nblk2, (unsigned)max_tiles, (unsigned)splits);
    dymoe_launch(ctx, DYMOE_K_GEMM2, (gemm_kernel<2>), g2, dim3(kGmThreads), kLdsBytes, st, xb, xh, hbuf,
                 bits, table, plan, P, E, k, H, F, (uint16_t*)nullptr, opair);
    DYMOE_HIP_LAUNCH_CHECK();
    const long n4 = (long)T * (H / 4);
    dymoe_launch(ctx, DYMOE_K_GEMM_COMBINE, gemm_combine_kernel, dim3((unsigned)((n4 + 255) / 256)), dim3(256), 0, st, opair,
                       idx, w, bits, T, H, E, k, splits, out_dtype, y);
    DYMOE_HIP_LAUNCH_CHECK();
    return DYMOE_OK;
}

}  // namespace dymoe
