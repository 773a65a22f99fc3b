// Decode path of the mixed-precision SwiGLU expert FFN: bandwidth-bound
// dequant-fused GEMV in two launches: phase 1 (gate and up projections, SwiGLU;
// one (token, expert) pair per grid row) and phase 2 (down projection of every
// expert of a token, weighted by the gate and summed into y).
//
// A wavefront streams weight rows.  A row is cut into segments of 2048
// columns; in a segment every lane owns a fixed set of 32 columns, so the
// activations a lane needs never change while it streams rows: they are
// loaded once into registers (packed pairs) and the weight stream is the only
// memory traffic of the loop.
//   bf16 rows : 4 x 16-byte loads per lane and segment, bf16 dot2 (phase 1)
//               or fp32 FMA (phase 2, fp32 intermediate)
//   int8 rows : two 16-byte loads per lane and segment (32 codes = half a group)
//   int4 rows : one 16-byte load per lane and segment (32 codes = half a group)
//   int2 rows : one  8-byte load per lane and segment (32 codes = half a group)
// The row loop is software pipelined: the loads of the next batch of rows are
// issued before the current batch is reduced, and every load is unconditional
// (lanes past the end of a row re-read the row's tail against zero
// activations) so that the loop body is straight-line code.
//
// Quantised codes are turned into fp16 without integer->float conversions:
// OR-ing a code field into the mantissa of 2^n (n chosen so that the field's
// lowest bit weighs 1) gives the fp16 number 2^n + q.  The dot product with
// the activations then runs on fp16 dot2 (fp32 accumulate) and the 2^n * x
// terms are removed with one precomputed constant per lane:
//   sum_k (s q_k + m) x_k = s * (sum_k (2^n_k + q_k) x_k - sum_k 2^n_k x_k) + m * sum_k x_k.
#include <math.h>

#include "common.hpp"
#include "assign.hpp"
#include "ffn_layout.hpp"
#include "route_device.hpp"

namespace dymoe {

constexpr int kGvThreads = 256;
constexpr int kGvWaves = kGvThreads / kWave;

// ------------------------------------------------------------------ activations

// 32 activations of one lane (quantised layouts), as fp16 pairs ordered for
// the code extraction below, plus the two per-lane constants.
struct LaneX {
    uint32_t r[16];
    float xsum;  // sum of the 64 activations of the lane's quantisation group (the lane's 32 and its partner's)
    float xoff;  // sum of 2^n_k * x_k
};

__device__ __forceinline__ float h2f(_Float16 h) { return (float)h; }

// v[32] are the lane's activations in column order.
template <int BITS>
__device__ __forceinline__ void arrange_lane_x(const float* v, LaneX& lx)
{
    _Float16 hv[32];
    float sum = 0.0f;
#pragma unroll
    for (int i = 0; i < 32; i++) {
        hv[i] = (_Float16)v[i];
        sum += h2f(hv[i]);
    }
    lx.xsum = sum + dpp_get<0xB1, 0xF>(sum);       // quad_perm [1,0,3,2]: lanes 2i and 2i+1 share a group
    float off = 0.0f;
    if (BITS == 8) {
        // dword d holds codes 4d..4d+3, one per byte; pairs (b0,b1) and (b2,b3), all offset by 1024
#pragma unroll
        for (int i = 0; i < 16; i++) {
            half2_t pr = {hv[2 * i], hv[2 * i + 1]};
            lx.r[i] = __builtin_bit_cast(uint32_t, pr);
        }
        off = 1024.0f * sum;
    } else if (BITS == 4) {
        // dword d holds codes 8d..8d+7 in nibbles 0..7
        // pairs: (n0,n4)+1024, (n1,n5)+64, (n2,n6)+1024, (n3,n7)+64
#pragma unroll
        for (int d = 0; d < 4; d++) {
#pragma unroll
            for (int j = 0; j < 4; j++) {
                const _Float16 a = hv[8 * d + j], b = hv[8 * d + 4 + j];
                half2_t pr = {a, b};
                lx.r[4 * d + j] = __builtin_bit_cast(uint32_t, pr);
                const float wgt = (j & 1) ? 64.0f : 1024.0f;
                off += wgt * (h2f(a) + h2f(b));
            }
        }
    } else {
        // dword d holds codes 16d..16d+15 in 2-bit fields 0..15; pair j = (field j, field 8+j)
        // offsets by field position: 1024, 256, 64, 16, 4, then (after >>10) 1024, 256, 64
        const float wgt[8] = {1024.0f, 256.0f, 64.0f, 16.0f, 4.0f, 1024.0f, 256.0f, 64.0f};
#pragma unroll
        for (int d = 0; d < 2; d++) {
#pragma unroll
            for (int j = 0; j < 8; j++) {
                const _Float16 a = hv[16 * d + j], b = hv[16 * d + 8 + j];
                half2_t pr = {a, b};
                lx.r[8 * d + j] = __builtin_bit_cast(uint32_t, pr);
                off += wgt[j] * (h2f(a) + h2f(b));
            }
        }
    }
    lx.xoff = off;
}

// sum_k (2^n_k + q_k) x_k over the lane's 32 int4 codes (one uint4)
__device__ __forceinline__ float dot_q4(const uint4 c, const LaneX& lx)
{
    const uint32_t w[4] = {c.x, c.y, c.z, c.w};
    float acc = 0.0f;
#pragma unroll
    for (int d = 0; d < 4; d++) {
        const uint32_t v = w[d], v8 = w[d] >> 8;
        acc = dot2_f16(and_or(v, 0x000F000Fu, 0x64006400u), lx.r[4 * d + 0], acc);
        acc = dot2_f16(and_or(v, 0x00F000F0u, 0x54005400u), lx.r[4 * d + 1], acc);
        acc = dot2_f16(and_or(v8, 0x000F000Fu, 0x64006400u), lx.r[4 * d + 2], acc);
        acc = dot2_f16(and_or(v8, 0x00F000F0u, 0x54005400u), lx.r[4 * d + 3], acc);
    }
    return acc;
}

// the same over the lane's 32 int2 codes (one uint2)
__device__ __forceinline__ float dot_q2(const uint2 c, const LaneX& lx)
{
    const uint32_t w[2] = {c.x, c.y};
    float acc = 0.0f;
#pragma unroll
    for (int d = 0; d < 2; d++) {
        const uint32_t v = w[d], v10 = w[d] >> 10;
        acc = dot2_f16(and_or(v, 0x00030003u, 0x64006400u), lx.r[8 * d + 0], acc);
        acc = dot2_f16(and_or(v, 0x000C000Cu, 0x5C005C00u), lx.r[8 * d + 1], acc);
        acc = dot2_f16(and_or(v, 0x00300030u, 0x54005400u), lx.r[8 * d + 2], acc);
        acc = dot2_f16(and_or(v, 0x00C000C0u, 0x4C004C00u), lx.r[8 * d + 3], acc);
        acc = dot2_f16(and_or(v, 0x03000300u, 0x44004400u), lx.r[8 * d + 4], acc);
        acc = dot2_f16(and_or(v10, 0x00030003u, 0x64006400u), lx.r[8 * d + 5], acc);
        acc = dot2_f16(and_or(v10, 0x000C000Cu, 0x5C005C00u), lx.r[8 * d + 6], acc);
        acc = dot2_f16(and_or(v10, 0x00300030u, 0x54005400u), lx.r[8 * d + 7], acc);
    }
    return acc;
}

// the same over the lane's 32 int8 codes (two uint4): a byte b becomes the fp16 number 1024 + b
__device__ __forceinline__ float dot_q8(const uint4 c0, const uint4 c1, const LaneX& lx)
{
    const uint32_t w[8] = {c0.x, c0.y, c0.z, c0.w, c1.x, c1.y, c1.z, c1.w};
    float acc = 0.0f;
#pragma unroll
    for (int d = 0; d < 8; d++) {
        acc = dot2_f16(__builtin_amdgcn_perm(0x64646464u, w[d], 0x04010400u), lx.r[2 * d], acc);
        acc = dot2_f16(__builtin_amdgcn_perm(0x64646464u, w[d], 0x04030402u), lx.r[2 * d + 1], acc);
    }
    return acc;
}

// activations of one lane for bf16 rows: NSEG x 4 chunks of 8, packed bf16 pairs
template <int NSEG>
struct LaneXB {
    uint4 r[NSEG][4];
};

// ------------------------------------------------------------------ weight rows

struct ExpertMat {
    const uint16_t* w;      // bf16
    const uint8_t* q;       // packed codes at the expert's precision
    const uint16_t* s;      // fp16 scale
    const uint16_t* z;      // fp16 zero
};

__device__ __forceinline__ ExpertMat pick_mat(const dymoe_expert_fmt& ex, int mat, int b)
{
    ExpertMat m;
    m.w = reinterpret_cast<const uint16_t*>(ex.w[mat]);
    if (b == 8) {
        m.q = ex.q8[mat];
        m.s = reinterpret_cast<const uint16_t*>(ex.s8[mat]);
        m.z = reinterpret_cast<const uint16_t*>(ex.z8[mat]);
    } else if (b == 4) {
        m.q = ex.q4[mat];
        m.s = reinterpret_cast<const uint16_t*>(ex.s4[mat]);
        m.z = reinterpret_cast<const uint16_t*>(ex.z4[mat]);
    } else {
        m.q = ex.q2[mat];
        m.s = reinterpret_cast<const uint16_t*>(ex.s2[mat]);
        m.z = reinterpret_cast<const uint16_t*>(ex.z2[mat]);
    }
    return m;
}

// Whether the table held the pointers of this matrix at b bits.  The bit widths are chosen on the device, so only the
// kernels can tell that an assigned format is absent; they test exactly the pointers they are about to read through.
__device__ __forceinline__ bool mat_present(const ExpertMat& m, int b)
{
    return (b == 16) ? (m.w != nullptr) : (m.q != nullptr && m.s != nullptr && m.z != nullptr);
}

// what one lane loads of one row: NSEG segments starting at column seg0 * 2048
template <int BITS, int NSEG> struct RowRegs;
template <int NSEG> struct RowRegs<16, NSEG> { uint4 c[NSEG][4]; };
template <int NSEG> struct RowRegs<4, NSEG> { uint4 c[NSEG]; uint16_t sz[NSEG]; };
template <int NSEG> struct RowRegs<2, NSEG> { uint2 c[NSEG]; uint16_t sz[NSEG]; };
template <int NSEG> struct RowRegs<8, NSEG> { uint4 c[NSEG][2]; uint16_t sz[NSEG]; };

// Issue the loads of row `row` (K columns).  Lanes past the end of the row
// re-read its tail: finite weights against zero activations add nothing.
// Weights are read once per step: where a load instruction covers whole cache
// lines (consecutive lanes, consecutive 16 or 8 bytes) it is marked non-temporal.
template <int BITS, int NSEG>
__device__ __forceinline__ void load_row(const ExpertMat& m, long row, int K, int seg0, int lane,
                                         RowRegs<BITS, NSEG>& rr)
{
    if constexpr (BITS == 16) {
        const uint16_t* base = m.w + row * K;
#pragma unroll
        for (int s = 0; s < NSEG; s++)
#pragma unroll
            for (int j = 0; j < 4; j++) {
                const int col = min((seg0 + s) * kSeg + (j * kWave + lane) * 8, K - 8);
                rr.c[s][j] = load_global_nt<uint4>(base + col);
            }
    } else {
        const long G = K >> 6;
        const uint8_t* codes = m.q + row * ((long)K * BITS / 8);
#pragma unroll
        for (int s = 0; s < NSEG; s++) {
            const int col0 = min((seg0 + s) * kSeg + 32 * lane, K - 32);
            if constexpr (BITS == 8) {
                // (ordinary loads: the two pieces of a lane interleave with its neighbours', and only a
                // cached line serves both)
                rr.c[s][0] = load_global<uint4>(codes + col0);
                rr.c[s][1] = load_global<uint4>(codes + col0 + 16);
            } else if constexpr (BITS == 4) rr.c[s] = load_global_nt<uint4>(codes + (col0 >> 1));
            else rr.c[s] = load_global_nt<uint2>(codes + (col0 >> 2));
            // the two lanes of a group share its scale and zero: the even lane fetches the scale, the odd one the
            // zero (one load instruction for both; dot_row_q puts the halves together)
            rr.sz[s] = load_global<uint16_t>(((lane & 1) ? m.z : m.s) + row * G + (col0 >> 6));
        }
    }
}

// per-lane partial dot product of a loaded quantised row
template <int BITS, int NSEG>
__device__ __forceinline__ float dot_row_q(const RowRegs<BITS, NSEG>& rr, const LaneX (&lx)[NSEG])
{
    float part = 0.0f;
#pragma unroll
    for (int s = 0; s < NSEG; s++) {
        float acc;
        if constexpr (BITS == 8) acc = dot_q8(rr.c[s][0], rr.c[s][1], lx[s]);
        else if constexpr (BITS == 4) acc = dot_q4(rr.c[s], lx[s]);
        else acc = dot_q2(rr.c[s], lx[s]);
        // group total = scale * sum_k q_k x_k + zero * sum_k x_k over both lanes' halves: the even lane, which holds
        // the scale, takes the first term (its partner's sum comes over by DPP), the odd lane the second
        const float qx = acc - lx[s].xoff;
        const float qx_group = qx + dpp_get<0xB1, 0xF>(qx);
        const float coef = h2f(f16_from_bits(rr.sz[s]));
        part += coef * ((threadIdx.x & 1) ? lx[s].xsum : qx_group);
    }
    return part;
}

// bf16 row against bf16 activations (exact products, fp32 accumulation)
template <int NSEG>
__device__ __forceinline__ float dot_row_b(const RowRegs<16, NSEG>& rr, const LaneXB<NSEG>& lx)
{
    float a = 0.0f;
#pragma unroll
    for (int s = 0; s < NSEG; s++)
#pragma unroll
        for (int j = 0; j < 4; j++) {
            a = dot2_bf16(rr.c[s][j].x, lx.r[s][j].x, a);
            a = dot2_bf16(rr.c[s][j].y, lx.r[s][j].y, a);
            a = dot2_bf16(rr.c[s][j].z, lx.r[s][j].z, a);
            a = dot2_bf16(rr.c[s][j].w, lx.r[s][j].w, a);
        }
    return a;
}

// ---------------------------------------------------------------- phase 1
// h[p,f] = silu(W1[f,:] . x_t) * (W3[f,:] . x_t)
// A wavefront takes RF consecutive f per iteration (2*RF rows in flight).

template <int BITS> struct Phase1Rows { static constexpr int RF = (BITS == 16) ? 1 : (BITS == 2 ? 4 : 2); };

template <int BITS, int NSEG, typename XT, typename DotFn>
__device__ __forceinline__ void phase1_rows(const ExpertMat& m1, const ExpertMat& m3, int H,
                                            int f_begin, int f_end, float* __restrict__ hrow,
                                            const XT& lx, DotFn dot)
{
    constexpr int RF = Phase1Rows<BITS>::RF;
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = threadIdx.x / kWave;
    // two register sets used in turn (the loop body handles two batches), so that a batch requested one pass
    // ahead is consumed where it landed: no copying from a "next" set to a "current" one
    RowRegs<BITS, NSEG> ra[2 * RF], rb[2 * RF];
    int f = f_begin + wave * RF;
    if (f >= f_end) return;
    constexpr int kStep = kGvWaves * RF;
    auto fetch = [&](RowRegs<BITS, NSEG>(&dst)[2 * RF], int f0) {   // rows clamped to the block's last row
#pragma unroll
        for (int i = 0; i < RF; i++) {
            const int fi = min(f0 + i, f_end - 1);
            load_row<BITS, NSEG>(m1, fi, H, 0, lane, dst[2 * i]);
            load_row<BITS, NSEG>(m3, fi, H, 0, lane, dst[2 * i + 1]);
        }
    };
    auto finish = [&](const RowRegs<BITS, NSEG>(&src)[2 * RF], int f0) {
        float a[RF], g[RF];
#pragma unroll
        for (int i = 0; i < RF; i++) {
            a[i] = dot(src[2 * i], lx);
            g[i] = dot(src[2 * i + 1], lx);
        }
#pragma unroll
        for (int i = 0; i < RF; i++) {
            a[i] = wave_sum_dpp(a[i]);
            g[i] = wave_sum_dpp(g[i]);
        }
        // lane i writes row f0 + i
        float hv = 0.0f;
#pragma unroll
        for (int i = 0; i < RF; i++)
            if (lane == i) hv = a[i] / (1.0f + __expf(-a[i])) * g[i];
        if (lane < RF && f0 + lane < f_end) hrow[f0 + lane] = hv;
    };
    fetch(ra, f);
    if constexpr (BITS >= 8) {
        for (; f < f_end; f += 2 * kStep) {
            fetch(rb, f + kStep);                    // next batch first
            finish(ra, f);
            if (f + kStep >= f_end) break;           // the same in every lane of the wavefront
            fetch(ra, f + 2 * kStep);
            finish(rb, f + kStep);
        }
    } else {
        // int4 / int2: four and eight rows per batch make the doubled loop body long enough to cost more in
        // instruction fetch than the copies it saves (measured: 24.5 against 22.6 us on the int2 pair)
        for (; f < f_end; f += kStep) {
            fetch(rb, f + kStep);
            finish(ra, f);
#pragma unroll
            for (int i = 0; i < 2 * RF; i++) ra[i] = rb[i];
        }
    }
}

template <int BITS, int NSEG, typename Missing>
__device__ __forceinline__ void phase1_quant(const ExpertMat& m1, const ExpertMat& m3,
                                             const uint16_t* __restrict__ xrow, int H, int f_begin,
                                             int f_end, float* __restrict__ hrow, Missing missing)
{
    const int lane = threadIdx.x & (kWave - 1);
    LaneX lx[NSEG];
#pragma unroll
    for (int s = 0; s < NSEG; s++) {
        float v[32];
        const int col0 = s * kSeg + 32 * lane;
#pragma unroll
        for (int c = 0; c < 4; c++) {
            uint4 raw = make_uint4(0, 0, 0, 0);
            if (col0 < H) raw = *reinterpret_cast<const uint4*>(xrow + col0 + 8 * c);
            v[8 * c + 0] = bf16_lo(raw.x); v[8 * c + 1] = bf16_hi(raw.x);
            v[8 * c + 2] = bf16_lo(raw.y); v[8 * c + 3] = bf16_hi(raw.y);
            v[8 * c + 4] = bf16_lo(raw.z); v[8 * c + 5] = bf16_hi(raw.z);
            v[8 * c + 6] = bf16_lo(raw.w); v[8 * c + 7] = bf16_hi(raw.w);
        }
        arrange_lane_x<BITS>(v, lx[s]);
    }
    // (tested here and not before the loads above: the table's pointers and the activations then arrive together)
    if (!mat_present(m1, BITS) || !mat_present(m3, BITS)) return missing();
    phase1_rows<BITS, NSEG>(m1, m3, H, f_begin, f_end, hrow, lx,
                            [](const RowRegs<BITS, NSEG>& rr, const LaneX (&l)[NSEG]) {
                                return dot_row_q<BITS, NSEG>(rr, l);
                            });
}

template <int NSEG, typename Missing>
__device__ __forceinline__ void phase1_bf16(const ExpertMat& m1, const ExpertMat& m3,
                                            const uint16_t* __restrict__ xrow, int H, int f_begin,
                                            int f_end, float* __restrict__ hrow, Missing missing)
{
    const int lane = threadIdx.x & (kWave - 1);
    LaneXB<NSEG> lx;
#pragma unroll
    for (int s = 0; s < NSEG; s++)
#pragma unroll
        for (int j = 0; j < 4; j++) {
            const int col = s * kSeg + (j * kWave + lane) * 8;
            lx.r[s][j] = make_uint4(0, 0, 0, 0);
            if (col < H) lx.r[s][j] = *reinterpret_cast<const uint4*>(xrow + col);
        }
    if (!mat_present(m1, 16) || !mat_present(m3, 16)) return missing();
    phase1_rows<16, NSEG>(m1, m3, H, f_begin, f_end, hrow, lx,
                          [](const RowRegs<16, NSEG>& rr, const LaneXB<NSEG>& l) {
                              return dot_row_b<NSEG>(rr, l);
                          });
}

// One (token, expert) pair p: rows [f_begin, f_end) of W1 and W3 of expert e at b bits.
template <int NSEG>
__device__ __forceinline__ void phase1_pair(const uint16_t* __restrict__ x, const dymoe_expert_fmt* __restrict__ table,
                                            int p, int e, int b, int H, int F, int k, int rows_per_block,
                                            float* __restrict__ hbuf, unsigned* __restrict__ flags)
{
    const int t = p / k;
    const int f_begin = blockIdx.x * rows_per_block;
    const int f_end = min(F, f_begin + rows_per_block);
    const uint16_t* xrow = x + (long)t * H;
    float* hrow = hbuf + (long)p * F;
    const dymoe_expert_fmt ex = table[e];
    // The assigned format may be absent from the table: the pair then contributes nothing.  Its rows of the
    // intermediate are set to zero, so that the second phase adds nothing for it even where it finds the down projection.
    auto missing = [&]() {
        for (int f = f_begin + (int)threadIdx.x; f < f_end; f += kGvThreads) hrow[f] = 0.0f;
        if (blockIdx.x == 0 && threadIdx.x == 0) atomicOr(flags, DYMOE_FLAG_FORMAT_MISSING);
    };
    if (b == 16) {
        phase1_bf16<NSEG>(pick_mat(ex, 0, 16), pick_mat(ex, 1, 16), xrow, H, f_begin, f_end, hrow, missing);
    } else if (b == 8) {
        phase1_quant<8, NSEG>(pick_mat(ex, 0, 8), pick_mat(ex, 1, 8), xrow, H, f_begin, f_end, hrow, missing);
    } else if (b == 4) {
        phase1_quant<4, NSEG>(pick_mat(ex, 0, 4), pick_mat(ex, 1, 4), xrow, H, f_begin, f_end, hrow, missing);
    } else {
        phase1_quant<2, NSEG>(pick_mat(ex, 0, 2), pick_mat(ex, 1, 2), xrow, H, f_begin, f_end, hrow, missing);
    }
}

template <int NSEG>
__global__ __launch_bounds__(kGvThreads) void gemv_phase1_kernel(
    const uint16_t* __restrict__ x, const int32_t* __restrict__ idx,
    const uint8_t* __restrict__ bits, const dymoe_expert_fmt* __restrict__ table, int H, int F,
    int E, int k, int rows_per_block, float* __restrict__ hbuf, unsigned* __restrict__ flags)
{
    // pairs in reverse: a token's later slots carry the less important experts, hence the narrower formats,
    // whose workgroups are short and latency-bound; dispatched first they overlap the wide ones instead of forming the tail
    const int p = (int)gridDim.y - 1 - (int)blockIdx.y;
    const int e = idx[p];
    if (e < 0 || e >= E) return;
    const int b = bits[e];
    if (b != 16 && b != 8 && b != 4 && b != 2) return;
    phase1_pair<NSEG>(x, table, p, e, b, H, F, k, rows_per_block, hbuf, flags);
}

// The first phase with the decode step's front end in front of it (router gating and top-k, decode importance,
// bit-width assignment: the arithmetic of dymoe_decode_front, same device functions, same order of every sum, so the
// same bits).  Every workgroup works the front end out for itself, in LDS, from the router (64 KiB for 8 experts of
// 4096: read from L2 by all but the first workgroups) and goes on to its rows without a launch boundary and without
// the chain of dependent loads (pair -> expert -> bit width) the stand-alone kernel starts with; workgroup (0, 0)
// also writes the front end's outputs to memory for the second phase and for the caller.
// Limits (checked by the launcher): T <= kFusedMaxTokens, E <= 64, k <= kFusedMaxK.
constexpr int kFusedMaxTokens = 4, kFusedMaxK = 8, kFusedMaxE = 64;

template <int NSEG, int NCH>
__global__ __launch_bounds__(kGvThreads) void decode_fused_phase1_kernel(
    const uint16_t* __restrict__ x, const uint16_t* __restrict__ wg, const float* __restrict__ bias,
    const dymoe_expert_fmt* __restrict__ table, int T, int H, int F, int E, int k, int renorm, TierTable tiers,
    int floor_bits, int rows_per_block, int32_t* __restrict__ idx, float* __restrict__ w, float* __restrict__ probs,
    float* __restrict__ importance, int32_t* __restrict__ load, uint8_t* __restrict__ bits,
    int32_t* __restrict__ rank, float* __restrict__ hbuf, unsigned* __restrict__ flags)
{
    __shared__ float s_logit[kFusedMaxE];
    __shared__ float s_selp[kFusedMaxK];
    __shared__ float s_imp[kFusedMaxE];
    __shared__ int32_t s_load[kFusedMaxE];
    __shared__ int32_t s_idx[kFusedMaxTokens * kFusedMaxK];
    __shared__ float s_w[kFusedMaxTokens * kFusedMaxK];
    __shared__ float s_probs[kFusedMaxTokens * kFusedMaxE];
    __shared__ uint8_t s_bits[kFusedMaxE];
    __shared__ int32_t s_rank[kFusedMaxE];
    const int wave = threadIdx.x / kWave;
    for (int e = threadIdx.x; e < E; e += kGvThreads) {
        s_imp[e] = 0.0f;
        s_load[e] = 0;
    }
    for (int t = 0; t < T; t++) {
        route_logits<1, NCH, kGvWaves>(x, wg, bias, T, H, E, t, s_logit);
        __syncthreads();
        if (wave == 0) route_select_fixed<1>(s_logit, s_selp, t, E, k, renorm, s_idx, s_w, s_probs, s_imp, s_load);
        __syncthreads();
    }
    for (int e = threadIdx.x; e < E; e += kGvThreads) {
        const float g = s_imp[e];
        s_imp[e] = (T <= 1) ? g : g / (float)T;
    }
    __syncthreads();
    assign_all<float>(kGvThreads, E, s_imp, s_load, tiers, floor_bits, s_bits, s_rank);
    __syncthreads();
    if (blockIdx.x == 0 && blockIdx.y == 0) {
        for (int i = threadIdx.x; i < T * k; i += kGvThreads) {
            idx[i] = s_idx[i];
            w[i] = s_w[i];
        }
        if (probs)
            for (int i = threadIdx.x; i < T * E; i += kGvThreads) probs[i] = s_probs[i];
        for (int e = threadIdx.x; e < E; e += kGvThreads) {
            importance[e] = s_imp[e];
            load[e] = s_load[e];
            bits[e] = s_bits[e];
            if (rank) rank[e] = s_rank[e];
        }
    }
    const int p = (int)gridDim.y - 1 - (int)blockIdx.y;
    const int e = s_idx[p];
    const int b = s_bits[e];
    if (b != 16 && b != 8 && b != 4 && b != 2) return;
    phase1_pair<NSEG>(x, table, p, e, b, H, F, k, rows_per_block, hbuf, flags);
}

// ---------------------------------------------------------------- phase 2
// y[t,j] = sum_slot w[t,slot] * sum_f W2_e[j,f] * h[p,f],  p = t*k + slot, e = idx[p]
// A workgroup owns kP2Rows consecutive rows j of one token, over every slot and every 2048-column segment of F:
// the (slot, segment) units are dealt out to its wavefronts.  A wavefront keeps the activations of its unit in
// registers, streams the unit's piece of every row and adds gate * partial into per-lane, per-row accumulators;
// only after its last unit are the accumulators summed over the lanes (once per row instead of once per row and
// segment), then over the wavefronts through LDS in a fixed order, and y is written: no partial sums in memory
// and no separate combining launch.

template <int BITS> struct Phase2Rows { static constexpr int R = (BITS == 16 || BITS == 8) ? 4 : 8; };

constexpr int kP2Rows = 16;
constexpr int kP2MaxWaves = 8;

// fp32 intermediate against bf16 weights
struct LaneH {
    float v[4][8];
};

__device__ __forceinline__ float dot_row_h(const RowRegs<16, 1>& rr, const LaneH& lh)
{
    float acc = 0.0f;
#pragma unroll
    for (int c = 0; c < 4; c++) {
        const uint4 u = rr.c[0][c];
        acc = fmaf(bf16_lo(u.x), lh.v[c][0], acc); acc = fmaf(bf16_hi(u.x), lh.v[c][1], acc);
        acc = fmaf(bf16_lo(u.y), lh.v[c][2], acc); acc = fmaf(bf16_hi(u.y), lh.v[c][3], acc);
        acc = fmaf(bf16_lo(u.z), lh.v[c][4], acc); acc = fmaf(bf16_hi(u.z), lh.v[c][5], acc);
        acc = fmaf(bf16_lo(u.w), lh.v[c][6], acc); acc = fmaf(bf16_hi(u.w), lh.v[c][7], acc);
    }
    return acc;
}

// one unit: segment `seg` of rows j_begin .. j_begin + kP2Rows - 1 (clamped to the last row H - 1)
template <int BITS, typename XT, typename DotFn>
__device__ __forceinline__ void phase2_unit(const ExpertMat& m2, int F, int seg, int j_begin, int H,
                                            float gate, float (&tot)[kP2Rows], const XT& lx, DotFn dot)
{
    constexpr int R = Phase2Rows<BITS>::R;
    constexpr int NB = kP2Rows / R;                 // 4 or 2 batches of rows
    static_assert(NB % 2 == 0, "batches come in pairs");
    const int lane = threadIdx.x & (kWave - 1);
    RowRegs<BITS, 1> ra[R], rb[R];                  // used in turn, as in phase 1
    auto fetch = [&](RowRegs<BITS, 1>(&dst)[R], int j0) {
#pragma unroll
        for (int i = 0; i < R; i++) load_row<BITS, 1>(m2, min(j0 + i, H - 1), F, seg, lane, dst[i]);
    };
    fetch(ra, j_begin);
#pragma unroll
    for (int bt = 0; bt < NB; bt += 2) {
        fetch(rb, j_begin + (bt + 1) * R);          // next batch first
#pragma unroll
        for (int i = 0; i < R; i++) tot[bt * R + i] = fmaf(gate, dot(ra[i], lx), tot[bt * R + i]);
        if (bt + 2 < NB) fetch(ra, j_begin + (bt + 2) * R);
#pragma unroll
        for (int i = 0; i < R; i++) tot[(bt + 1) * R + i] = fmaf(gate, dot(rb[i], lx), tot[(bt + 1) * R + i]);
    }
}

// Two units of narrow formats (int4, int2) side by side: a wavefront's start-up chain (pair -> expert -> bit width ->
// table entry -> activations -> first rows) is a string of dependent latencies, and with 16 rows of int4 or int2
// there is little streaming to hide the second unit's chain behind.  Taken together, both chains run at once.
template <int BA, int BB>
__device__ __forceinline__ void phase2_two_units(const ExpertMat& ma, const ExpertMat& mb, int F, int sa, int sb,
                                                 int j_begin, int H, float ga, float gb,
                                                 float (&tot)[kP2Rows], const LaneX (&la)[1], const LaneX (&lb)[1])
{
    constexpr int R = (BA == 2 && BB == 2) ? 8 : 4;
    constexpr int NB = kP2Rows / R;
    static_assert(NB % 2 == 0, "batches come in pairs");
    const int lane = threadIdx.x & (kWave - 1);
    RowRegs<BA, 1> a0[R], a1[R];
    RowRegs<BB, 1> b0[R], b1[R];
    auto fetch = [&](RowRegs<BA, 1>(&da)[R], RowRegs<BB, 1>(&db)[R], int j0) {
#pragma unroll
        for (int i = 0; i < R; i++) {
            const int row = min(j0 + i, H - 1);
            load_row<BA, 1>(ma, row, F, sa, lane, da[i]);
            load_row<BB, 1>(mb, row, F, sb, lane, db[i]);
        }
    };
    auto finish = [&](const RowRegs<BA, 1>(&da)[R], const RowRegs<BB, 1>(&db)[R], int bt) {
#pragma unroll
        for (int i = 0; i < R; i++) {
            float acc = fmaf(ga, dot_row_q<BA, 1>(da[i], la), tot[bt * R + i]);
            tot[bt * R + i] = fmaf(gb, dot_row_q<BB, 1>(db[i], lb), acc);
        }
    };
    fetch(a0, b0, j_begin);
#pragma unroll
    for (int bt = 0; bt < NB; bt += 2) {
        fetch(a1, b1, j_begin + (bt + 1) * R);
        finish(a0, b0, bt);
        if (bt + 2 < NB) fetch(a0, b0, j_begin + (bt + 2) * R);
        finish(a1, b1, bt + 1);
    }
}

__global__ __launch_bounds__(kP2MaxWaves * kWave) void gemv_phase2_kernel(
    const float* __restrict__ hbuf, const int32_t* __restrict__ idx, const float* __restrict__ w,
    const uint8_t* __restrict__ bits, const dymoe_expert_fmt* __restrict__ table, int H, int F,
    int E, int k, int nseg, int out_dtype, void* __restrict__ y, unsigned* __restrict__ flags)
{
    __shared__ float s_red[kP2MaxWaves][kP2Rows];
    const int t = blockIdx.y;
    const int j_begin = blockIdx.x * kP2Rows;
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
    const int nwaves = blockDim.x / kWave;
    float tot[kP2Rows];
#pragma unroll
    for (int i = 0; i < kP2Rows; i++) tot[i] = 0.0f;
    const int units = k * nseg;
    const int rounds = (units + nwaves - 1) / nwaves;
    // odd wavefronts take their units in reverse: the slots of a token differ in format (the later, the narrower),
    // and a compute unit should at any time hold wavefronts on wide, bandwidth-bound rows beside wavefronts on
    // narrow, instruction-bound ones instead of all of them on the same kind
    struct Unit {
        int valid, p, s, e, b;
    };
    auto unit_of = [&](int r) {
        Unit un = {0, 0, 0, 0, 0};
        if (r >= rounds) return un;
        const int u = wave + nwaves * ((wave & 1) ? rounds - 1 - r : r);
        if (u >= units) return un;
        const int slot = u / nseg;
        un.s = u - slot * nseg;
        un.p = t * k + slot;
        un.e = idx[un.p];
        if (un.e < 0 || un.e >= E) return un;       // pairs of skipped experts add nothing
        un.b = bits[un.e];
        un.valid = (un.b == 16 || un.b == 8 || un.b == 4 || un.b == 2);
        return un;
    };
    auto quant_x = [&](const Unit& un, float (&v)[32]) {
        const float* hrow = hbuf + (long)un.p * F;
        const int col0 = un.s * kSeg + 32 * lane;
#pragma unroll
        for (int c = 0; c < 8; c++) {
            float4 q = make_float4(0.f, 0.f, 0.f, 0.f);
            if (col0 < F) q = *reinterpret_cast<const float4*>(hrow + col0 + 4 * c);
            v[4 * c + 0] = q.x; v[4 * c + 1] = q.y; v[4 * c + 2] = q.z; v[4 * c + 3] = q.w;
        }
    };
    auto one_unit = [&](const Unit& un) {
        const int p = un.p, s = un.s, e = un.e, b = un.b;
        const float gate = w[p];
        const float* hrow = hbuf + (long)p * F;
        const dymoe_expert_fmt ex = table[e];
        auto missing = [&]() {                 // format not in the table: the pair is left out
            if (blockIdx.x == 0 && lane == 0) atomicOr(flags, DYMOE_FLAG_FORMAT_MISSING);
        };
        if (b == 16) {
            const ExpertMat m2 = pick_mat(ex, 2, 16);
            if (!mat_present(m2, 16)) return missing();
            LaneH lh;
#pragma unroll
            for (int c = 0; c < 4; c++) {
                const int col = s * kSeg + (c * kWave + lane) * 8;
#pragma unroll
                for (int i = 0; i < 8; i++) lh.v[c][i] = 0.0f;
                if (col < F) {
                    const float4 lo = *reinterpret_cast<const float4*>(hrow + col);
                    const float4 hi = *reinterpret_cast<const float4*>(hrow + col + 4);
                    lh.v[c][0] = lo.x; lh.v[c][1] = lo.y; lh.v[c][2] = lo.z; lh.v[c][3] = lo.w;
                    lh.v[c][4] = hi.x; lh.v[c][5] = hi.y; lh.v[c][6] = hi.z; lh.v[c][7] = hi.w;
                }
            }
            phase2_unit<16>(m2, F, s, j_begin, H, gate, tot, lh,
                            [](const RowRegs<16, 1>& rr, const LaneH& l) { return dot_row_h(rr, l); });
        } else {
            const ExpertMat m2 = (b == 8) ? pick_mat(ex, 2, 8) : (b == 4) ? pick_mat(ex, 2, 4) : pick_mat(ex, 2, 2);
            if (!mat_present(m2, b)) return missing();
            float v[32];
            quant_x(un, v);
            LaneX lx[1];
            if (b == 8) {
                arrange_lane_x<8>(v, lx[0]);
                phase2_unit<8>(m2, F, s, j_begin, H, gate, tot, lx,
                               [](const RowRegs<8, 1>& rr, const LaneX (&l)[1]) { return dot_row_q<8, 1>(rr, l); });
            } else if (b == 4) {
                arrange_lane_x<4>(v, lx[0]);
                phase2_unit<4>(m2, F, s, j_begin, H, gate, tot, lx,
                               [](const RowRegs<4, 1>& rr, const LaneX (&l)[1]) { return dot_row_q<4, 1>(rr, l); });
            } else {
                arrange_lane_x<2>(v, lx[0]);
                phase2_unit<2>(m2, F, s, j_begin, H, gate, tot, lx,
                               [](const RowRegs<2, 1>& rr, const LaneX (&l)[1]) { return dot_row_q<2, 1>(rr, l); });
            }
        }
    };
    for (int r = 0; r < rounds; r += 2) {
        const Unit ua = unit_of(r), ub = unit_of(r + 1);
        bool both = ua.valid && ub.valid && (ua.b == 4 || ua.b == 2) && (ub.b == 4 || ub.b == 2);
        ExpertMat ma = {}, mb = {};
        if (both) {
            ma = pick_mat(table[ua.e], 2, ua.b);
            mb = pick_mat(table[ub.e], 2, ub.b);
            both = mat_present(ma, ua.b) && mat_present(mb, ub.b);   // (if not: one by one, each tested again)
        }
        if (both) {
            const float ga = w[ua.p], gb = w[ub.p];
            LaneX la[1], lb[1];
            {
                float v[32];
                quant_x(ua, v);
                if (ua.b == 4) arrange_lane_x<4>(v, la[0]);
                else arrange_lane_x<2>(v, la[0]);
            }
            {
                float v[32];
                quant_x(ub, v);
                if (ub.b == 4) arrange_lane_x<4>(v, lb[0]);
                else arrange_lane_x<2>(v, lb[0]);
            }
            if (ua.b == 4 && ub.b == 4)
                phase2_two_units<4, 4>(ma, mb, F, ua.s, ub.s, j_begin, H, ga, gb, tot, la, lb);
            else if (ua.b == 4)
                phase2_two_units<4, 2>(ma, mb, F, ua.s, ub.s, j_begin, H, ga, gb, tot, la, lb);
            else if (ub.b == 4)
                phase2_two_units<2, 4>(ma, mb, F, ua.s, ub.s, j_begin, H, ga, gb, tot, la, lb);
            else
                phase2_two_units<2, 2>(ma, mb, F, ua.s, ub.s, j_begin, H, ga, gb, tot, la, lb);
        } else {
            if (ua.valid) one_unit(ua);
            if (ub.valid) one_unit(ub);
        }
    }
    // lanes, then wavefronts (in wavefront order: the result does not depend on timing)
    float o = 0.0f;
#pragma unroll
    for (int i = 0; i < kP2Rows; i++) {
        const float r = wave_sum_dpp(tot[i]);
        if (lane == i) o = r;
    }
    if (lane < kP2Rows) s_red[wave][lane] = o;
    __syncthreads();
    const int j = j_begin + (int)threadIdx.x;
    if (threadIdx.x < kP2Rows && j < H) {
        float acc = 0.0f;
        for (int wv = 0; wv < nwaves; wv++) acc += s_red[wv][threadIdx.x];
        const long i = (long)t * H + j;
        if (out_dtype == DYMOE_OUT_F32) reinterpret_cast<float*>(y)[i] = acc;
        else reinterpret_cast<uint16_t*>(y)[i] = (uint16_t)f32_to_bf16_bits(acc);
    }
}

// rows per workgroup of the first phase: 64 on the Mixtral-shaped decode layer (measured: beat 16..128), which makes 448
// workgroups; smaller layers get fewer rows per workgroup so that the launch still fills the chip
static int phase1_rows_per_block(long rows_total)
{
    int r = 64;
    while (r > 8 && rows_total / r < 384) r >>= 1;
    return r;
}

static int phase2_launch(dymoe_ctx* ctx, const float* hbuf, const int32_t* idx, const float* w, const uint8_t* bits,
                         const dymoe_expert_fmt* table, int T, int H, int F, int E, int k, int out_dtype, void* y,
                         hipStream_t st)
{
    // as many wavefronts as (slot, segment) units, at most kP2MaxWaves; of the counts that need the
    // fewest rounds the smallest, so that no wavefront idles through the last round
    const int nseg2 = (F + kSeg - 1) / kSeg;
    const int units = k * nseg2;
    int nwaves = units < kP2MaxWaves ? units : kP2MaxWaves;
    {
        const int rounds = (units + nwaves - 1) / nwaves;
        while (nwaves > 1 && (units + nwaves - 2) / (nwaves - 1) == rounds) nwaves--;
    }
    const dim3 g2((unsigned)((H + kP2Rows - 1) / kP2Rows), (unsigned)T);
    dymoe_launch(ctx, DYMOE_K_GEMV_PHASE2, gemv_phase2_kernel, g2, dim3((unsigned)(nwaves * kWave)), 0, st, hbuf, idx, w,
                 bits, table, H, F, E, k, nseg2, out_dtype, y, ctx->device_flags);
    DYMOE_HIP_LAUNCH_CHECK();
    return DYMOE_OK;
}

int ffn_gemv_launch(dymoe_ctx* ctx, const void* x, const int32_t* idx, const float* w,
                    const uint8_t* bits, const dymoe_expert_fmt* table, int T, int H, int F, int E,
                    int k, int out_dtype, void* y, void* workspace, hipStream_t st)
{
    const FfnLayout L = ffn_layout(T, H, F, E, k);
    float* hbuf = reinterpret_cast<float*>((char*)workspace + L.hbuf);
    const int P = T * k;
    const int nseg1 = (H + kSeg - 1) / kSeg;
    const int rows1 = phase1_rows_per_block((long)F * P);
    const dim3 g1((unsigned)((F + rows1 - 1) / rows1), (unsigned)P);
    const uint16_t* xb = (const uint16_t*)x;
    {
        switch (nseg1) {
        case 1: dymoe_launch(ctx, DYMOE_K_GEMV_PHASE1, (gemv_phase1_kernel<1>), g1, dim3(kGvThreads), 0, st, xb, idx, bits, table, H, F, E, k, rows1, hbuf, ctx->device_flags); break;
        case 2: dymoe_launch(ctx, DYMOE_K_GEMV_PHASE1, (gemv_phase1_kernel<2>), g1, dim3(kGvThreads), 0, st, xb, idx, bits, table, H, F, E, k, rows1, hbuf, ctx->device_flags); break;
        case 3: dymoe_launch(ctx, DYMOE_K_GEMV_PHASE1, (gemv_phase1_kernel<3>), g1, dim3(kGvThreads), 0, st, xb, idx, bits, table, H, F, E, k, rows1, hbuf, ctx->device_flags); break;
        case 4: dymoe_launch(ctx, DYMOE_K_GEMV_PHASE1, (gemv_phase1_kernel<4>), g1, dim3(kGvThreads), 0, st, xb, idx, bits, table, H, F, E, k, rows1, hbuf, ctx->device_flags); break;
        default: return DYMOE_ENOTSUP;
        }
    }
    DYMOE_HIP_LAUNCH_CHECK();
    return phase2_launch(ctx, hbuf, idx, w, bits, table, T, H, F, E, k, out_dtype, y, st);
}

// Whether the fused decode step covers these sizes.
bool decode_fused_fits(int T, int H, int E, int k)
{
    return T >= 1 && T <= kFusedMaxTokens && E <= kFusedMaxE && k <= kFusedMaxK && H % 64 == 0 && H <= 4 * kSeg;
}

int decode_fused_launch(dymoe_ctx* ctx, const void* x, const void* wg, const float* bias, const TierTable& tt,
                        int floor_bits, const dymoe_expert_fmt* table, int T, int H, int F, int E, int k, int renorm,
                        int out_dtype, int32_t* idx, float* w, float* probs, float* importance, int32_t* load,
                        uint8_t* bits, int32_t* rank, void* y, void* workspace, hipStream_t st)
{
    const FfnLayout L = ffn_layout(T, H, F, E, k);
    float* hbuf = reinterpret_cast<float*>((char*)workspace + L.hbuf);
    const int P = T * k;
    const int nseg1 = (H + kSeg - 1) / kSeg;
    const int rows1 = phase1_rows_per_block((long)F * P);
    const dim3 g1((unsigned)((F + rows1 - 1) / rows1), (unsigned)P);
    const uint16_t* xb = (const uint16_t*)x;
    const uint16_t* wb = (const uint16_t*)wg;
    // NCH: 16-byte chunks of an activation row per lane, as in dymoe_decode_front (8 up to 4096 columns, then 16)
#define DYMOE_FUSED(NSEG_, NCH_)                                                                                        \
    dymoe_launch(ctx, DYMOE_K_GEMV_PHASE1, (decode_fused_phase1_kernel<NSEG_, NCH_>), g1, dim3(kGvThreads), 0, st, xb, wb,  \
                 bias, table, T, H, F, E, k, renorm, tt, floor_bits, rows1, idx, w, probs, importance, load, bits, rank, hbuf,  \
                 ctx->device_flags)
    switch (nseg1) {
    case 1: DYMOE_FUSED(1, 8); break;
    case 2: DYMOE_FUSED(2, 8); break;
    case 3: DYMOE_FUSED(3, 16); break;
    case 4: DYMOE_FUSED(4, 16); break;
    default: return DYMOE_ENOTSUP;
    }
#undef DYMOE_FUSED
    DYMOE_HIP_LAUNCH_CHECK();
    return phase2_launch(ctx, hbuf, idx, w, bits, table, T, H, F, E, k, out_dtype, y, st);
}

}  // namespace dymoe
