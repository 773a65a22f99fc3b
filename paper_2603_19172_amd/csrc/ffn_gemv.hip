// Decode path of the mixed-precision SwiGLU expert FFN: bandwidth-bound
// dequant-fused GEMV, one (token, expert) pair per grid row.
//
// A wavefront owns whole weight rows.  A row is cut into segments of 2048
// columns; in a segment every lane owns a fixed set of 32 columns, so the
// activations a lane needs never change while it streams rows: they are
// loaded once into registers (packed pairs) and the weight stream is the only
// memory traffic of the loop.
//   bf16 rows : 4 x 16-byte loads per lane and segment, bf16 dot2 (phase 1)
//               or fp32 FMA (phase 2, fp32 intermediate)
//   int4 rows : one 16-byte load per lane and segment (32 codes = half a group)
//   int2 rows : one  8-byte load per lane and segment (32 codes = half a group)
// Quantised codes are turned into fp16 without integer->float conversions:
// OR-ing a code field into the mantissa of 2^n (n chosen so that the field's
// lowest bit weighs 1) gives the fp16 number 2^n + q.  The dot product with
// the activations then runs on fp16 dot2 (fp32 accumulate) and the 2^n * x
// terms are removed with one precomputed constant per lane:
//   sum_k (s q_k + m) x_k = s * (sum_k (2^n_k + q_k) x_k - sum_k 2^n_k x_k) + m * sum_k x_k.
#include <math.h>

#include "common.hpp"
#include "ffn_layout.hpp"

namespace dymoe {

constexpr int kGvThreads = 256;
constexpr int kGvWaves = kGvThreads / kWave;

// 32 activations of one lane (quantised layouts), as fp16 pairs ordered for
// the code extraction below, plus the two per-lane constants.
struct LaneX {
    uint32_t r[16];
    float xsum;  // sum of the lane's 32 activations
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
    lx.xsum = sum;
    float off = 0.0f;
    if (BITS == 4) {
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
        acc = dot2_f16((v & 0x000F000Fu) | 0x64006400u, lx.r[4 * d + 0], acc);
        acc = dot2_f16((v & 0x00F000F0u) | 0x54005400u, lx.r[4 * d + 1], acc);
        acc = dot2_f16((v8 & 0x000F000Fu) | 0x64006400u, lx.r[4 * d + 2], acc);
        acc = dot2_f16((v8 & 0x00F000F0u) | 0x54005400u, lx.r[4 * d + 3], acc);
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
        acc = dot2_f16((v & 0x00030003u) | 0x64006400u, lx.r[8 * d + 0], acc);
        acc = dot2_f16((v & 0x000C000Cu) | 0x5C005C00u, lx.r[8 * d + 1], acc);
        acc = dot2_f16((v & 0x00300030u) | 0x54005400u, lx.r[8 * d + 2], acc);
        acc = dot2_f16((v & 0x00C000C0u) | 0x4C004C00u, lx.r[8 * d + 3], acc);
        acc = dot2_f16((v & 0x03000300u) | 0x44004400u, lx.r[8 * d + 4], acc);
        acc = dot2_f16((v10 & 0x00030003u) | 0x64006400u, lx.r[8 * d + 5], acc);
        acc = dot2_f16((v10 & 0x000C000Cu) | 0x5C005C00u, lx.r[8 * d + 6], acc);
        acc = dot2_f16((v10 & 0x00300030u) | 0x54005400u, lx.r[8 * d + 7], acc);
    }
    return acc;
}

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
    if (b == 4) {
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

// per-lane partial of one quantised row over NSEG segments of a K-column row
template <int BITS, int NSEG>
__device__ __forceinline__ float qrow_partial(const ExpertMat& m, long row, int K, int lane,
                                              const LaneX (&lx)[NSEG])
{
    const long G = K >> 6;
    const uint8_t* codes = m.q + row * ((long)K * BITS / 8);
    float part = 0.0f;
#pragma unroll
    for (int s = 0; s < NSEG; s++) {
        const int col0 = s * kSeg + 32 * lane;
        if (col0 < K) {
            const long g = row * G + (col0 >> 6);
            const float sc = h2f(f16_from_bits(m.s[g]));
            const float zr = h2f(f16_from_bits(m.z[g]));
            float acc;
            if (BITS == 4) acc = dot_q4(*reinterpret_cast<const uint4*>(codes + (col0 >> 1)), lx[s]);
            else acc = dot_q2(*reinterpret_cast<const uint2*>(codes + (col0 >> 2)), lx[s]);
            part += sc * (acc - lx[s].xoff) + zr * lx[s].xsum;
        }
    }
    return part;
}

// ---------------------------------------------------------------- phase 1
// h[p,f] = silu(W1[f,:] . x_t) * (W3[f,:] . x_t)

template <int BITS, int NSEG>
__device__ __forceinline__ void phase1_quant(const ExpertMat& m1, const ExpertMat& m3,
                                             const uint16_t* __restrict__ xrow, int H, int f_begin,
                                             int f_end, float* __restrict__ hrow)
{
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = threadIdx.x / kWave;
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
    for (int f = f_begin + wave; f < f_end; f += kGvWaves) {
        float a = qrow_partial<BITS, NSEG>(m1, f, H, lane, lx);
        float g = qrow_partial<BITS, NSEG>(m3, f, H, lane, lx);
        a = wave_sum(a);
        g = wave_sum(g);
        if (lane == 0) hrow[f] = a / (1.0f + expf(-a)) * g;
    }
}

template <int NSEG>
__device__ __forceinline__ void phase1_bf16(const uint16_t* __restrict__ w1,
                                            const uint16_t* __restrict__ w3,
                                            const uint16_t* __restrict__ xrow, int H, int f_begin,
                                            int f_end, float* __restrict__ hrow)
{
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = threadIdx.x / kWave;
    uint4 xr[NSEG][4];
#pragma unroll
    for (int s = 0; s < NSEG; s++)
#pragma unroll
        for (int j = 0; j < 4; j++) {
            const int col = s * kSeg + (j * kWave + lane) * 8;
            xr[s][j] = make_uint4(0, 0, 0, 0);
            if (col < H) xr[s][j] = *reinterpret_cast<const uint4*>(xrow + col);
        }
    for (int f = f_begin + wave; f < f_end; f += kGvWaves) {
        const uint16_t* r1 = w1 + (long)f * H;
        const uint16_t* r3 = w3 + (long)f * H;
        float a = 0.0f, g = 0.0f;
#pragma unroll
        for (int s = 0; s < NSEG; s++)
#pragma unroll
            for (int j = 0; j < 4; j++) {
                const int col = s * kSeg + (j * kWave + lane) * 8;
                if (col < H) {
                    const uint4 u = *reinterpret_cast<const uint4*>(r1 + col);
                    const uint4 v = *reinterpret_cast<const uint4*>(r3 + col);
                    a = dot2_bf16(u.x, xr[s][j].x, a); a = dot2_bf16(u.y, xr[s][j].y, a);
                    a = dot2_bf16(u.z, xr[s][j].z, a); a = dot2_bf16(u.w, xr[s][j].w, a);
                    g = dot2_bf16(v.x, xr[s][j].x, g); g = dot2_bf16(v.y, xr[s][j].y, g);
                    g = dot2_bf16(v.z, xr[s][j].z, g); g = dot2_bf16(v.w, xr[s][j].w, g);
                }
            }
        a = wave_sum(a);
        g = wave_sum(g);
        if (lane == 0) hrow[f] = a / (1.0f + expf(-a)) * g;
    }
}

template <int NSEG>
__global__ __launch_bounds__(kGvThreads) void gemv_phase1_kernel(
    const uint16_t* __restrict__ x, const int32_t* __restrict__ idx,
    const uint8_t* __restrict__ bits, const dymoe_expert_fmt* __restrict__ table, int H, int F,
    int E, int k, int rows_per_block, float* __restrict__ hbuf)
{
    const int p = blockIdx.y;
    const int e = idx[p];
    if (e < 0 || e >= E) return;
    const int b = bits[e];
    if (b != 16 && b != 4 && b != 2) return;
    const int t = p / k;
    const int f_begin = blockIdx.x * rows_per_block;
    const int f_end = min(F, f_begin + rows_per_block);
    const uint16_t* xrow = x + (long)t * H;
    float* hrow = hbuf + (long)p * F;
    const dymoe_expert_fmt ex = table[e];
    if (b == 16) {
        phase1_bf16<NSEG>(reinterpret_cast<const uint16_t*>(ex.w[0]),
                          reinterpret_cast<const uint16_t*>(ex.w[1]), xrow, H, f_begin, f_end, hrow);
    } else if (b == 4) {
        phase1_quant<4, NSEG>(pick_mat(ex, 0, 4), pick_mat(ex, 1, 4), xrow, H, f_begin, f_end, hrow);
    } else {
        phase1_quant<2, NSEG>(pick_mat(ex, 0, 2), pick_mat(ex, 1, 2), xrow, H, f_begin, f_end, hrow);
    }
}

// ---------------------------------------------------------------- phase 2
// part[p,s,j] = sum over segment s of W2[j,f] * h[p,f]

__global__ __launch_bounds__(kGvThreads) void gemv_phase2_kernel(
    const float* __restrict__ hbuf, const int32_t* __restrict__ idx,
    const uint8_t* __restrict__ bits, const dymoe_expert_fmt* __restrict__ table, int H, int F,
    int E, int rows_per_block, int nseg, float* __restrict__ part)
{
    const int p = blockIdx.z;
    const int s = blockIdx.y;
    const int e = idx[p];
    if (e < 0 || e >= E) return;
    const int b = bits[e];
    if (b != 16 && b != 4 && b != 2) return;
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = threadIdx.x / kWave;
    const int j_begin = blockIdx.x * rows_per_block;
    const int j_end = min(H, j_begin + rows_per_block);
    const float* hrow = hbuf + (long)p * F;
    float* out = part + ((long)p * nseg + s) * H;
    const dymoe_expert_fmt ex = table[e];
    if (b == 16) {
        const uint16_t* w2 = reinterpret_cast<const uint16_t*>(ex.w[2]);
        float hr[4][8];
#pragma unroll
        for (int c = 0; c < 4; c++) {
            const int col = s * kSeg + (c * kWave + lane) * 8;
#pragma unroll
            for (int i = 0; i < 8; i++) hr[c][i] = 0.0f;
            if (col < F) {
                const float4 lo = *reinterpret_cast<const float4*>(hrow + col);
                const float4 hi = *reinterpret_cast<const float4*>(hrow + col + 4);
                hr[c][0] = lo.x; hr[c][1] = lo.y; hr[c][2] = lo.z; hr[c][3] = lo.w;
                hr[c][4] = hi.x; hr[c][5] = hi.y; hr[c][6] = hi.z; hr[c][7] = hi.w;
            }
        }
        for (int j = j_begin + wave; j < j_end; j += kGvWaves) {
            const uint16_t* row = w2 + (long)j * F;
            float acc = 0.0f;
#pragma unroll
            for (int c = 0; c < 4; c++) {
                const int col = s * kSeg + (c * kWave + lane) * 8;
                if (col < F) {
                    const uint4 u = *reinterpret_cast<const uint4*>(row + col);
                    acc = fmaf(bf16_lo(u.x), hr[c][0], acc); acc = fmaf(bf16_hi(u.x), hr[c][1], acc);
                    acc = fmaf(bf16_lo(u.y), hr[c][2], acc); acc = fmaf(bf16_hi(u.y), hr[c][3], acc);
                    acc = fmaf(bf16_lo(u.z), hr[c][4], acc); acc = fmaf(bf16_hi(u.z), hr[c][5], acc);
                    acc = fmaf(bf16_lo(u.w), hr[c][6], acc); acc = fmaf(bf16_hi(u.w), hr[c][7], acc);
                }
            }
            acc = wave_sum(acc);
            if (lane == 0) out[j] = acc;
        }
    } else {
        const ExpertMat m2 = pick_mat(ex, 2, b);
        const int col0 = s * kSeg + 32 * lane;
        float v[32];
#pragma unroll
        for (int c = 0; c < 8; c++) {
            float4 q = make_float4(0.f, 0.f, 0.f, 0.f);
            if (col0 < F) q = *reinterpret_cast<const float4*>(hrow + col0 + 4 * c);
            v[4 * c + 0] = q.x; v[4 * c + 1] = q.y; v[4 * c + 2] = q.z; v[4 * c + 3] = q.w;
        }
        LaneX lx;
        const long G = F >> 6;
        if (b == 4) {
            arrange_lane_x<4>(v, lx);
            for (int j = j_begin + wave; j < j_end; j += kGvWaves) {
                float acc = 0.0f;
                if (col0 < F) {
                    const long g = (long)j * G + (col0 >> 6);
                    const float sc = h2f(f16_from_bits(m2.s[g]));
                    const float zr = h2f(f16_from_bits(m2.z[g]));
                    const float d = dot_q4(*reinterpret_cast<const uint4*>(m2.q + (long)j * (F >> 1) + (col0 >> 1)), lx);
                    acc = sc * (d - lx.xoff) + zr * lx.xsum;
                }
                acc = wave_sum(acc);
                if (lane == 0) out[j] = acc;
            }
        } else {
            arrange_lane_x<2>(v, lx);
            for (int j = j_begin + wave; j < j_end; j += kGvWaves) {
                float acc = 0.0f;
                if (col0 < F) {
                    const long g = (long)j * G + (col0 >> 6);
                    const float sc = h2f(f16_from_bits(m2.s[g]));
                    const float zr = h2f(f16_from_bits(m2.z[g]));
                    const float d = dot_q2(*reinterpret_cast<const uint2*>(m2.q + (long)j * (F >> 2) + (col0 >> 2)), lx);
                    acc = sc * (d - lx.xoff) + zr * lx.xsum;
                }
                acc = wave_sum(acc);
                if (lane == 0) out[j] = acc;
            }
        }
    }
}

// y[t,j] = sum_slot w[t,slot] * sum_s part[p,s,j]   (pairs of skipped experts omitted)
__global__ __launch_bounds__(256) void gemv_combine_kernel(
    const float* __restrict__ part, const int32_t* __restrict__ idx,
    const float* __restrict__ w, const uint8_t* __restrict__ bits, int T, int H, int E, int k,
    int nseg, int out_dtype, void* __restrict__ y)
{
    const long i = (long)blockIdx.x * 256 + threadIdx.x;
    if (i >= (long)T * H) return;
    const int t = (int)(i / H);
    const int j = (int)(i - (long)t * H);
    float acc = 0.0f;
    for (int slot = 0; slot < k; slot++) {
        const int p = t * k + slot;
        const int e = idx[p];
        if (e < 0 || e >= E) continue;
        const int b = bits[e];
        if (b != 16 && b != 4 && b != 2) continue;
        float o = 0.0f;
        for (int s = 0; s < nseg; s++) o += part[((long)p * nseg + s) * H + j];
        acc = fmaf(w[p], o, acc);
    }
    if (out_dtype == DYMOE_OUT_F32) reinterpret_cast<float*>(y)[i] = acc;
    else reinterpret_cast<uint16_t*>(y)[i] = (uint16_t)f32_to_bf16_bits(acc);
}

int ffn_gemv_launch(dymoe_ctx* ctx, const void* x, const int32_t* idx, const float* w, const uint8_t* bits,
                    const dymoe_expert_fmt* table, int T, int H, int F, int E, int k,
                    int out_dtype, void* y, void* workspace, hipStream_t st)
{
    const FfnLayout L = ffn_layout(T, H, F, E, k);
    float* hbuf = reinterpret_cast<float*>((char*)workspace + L.hbuf);
    float* part = reinterpret_cast<float*>((char*)workspace + L.part);
    const int P = T * k;
    const int nseg1 = (H + kSeg - 1) / kSeg;
    const int nseg2 = (F + kSeg - 1) / kSeg;
    const int rows1 = 32, rows2 = 64;
    const dim3 g1((unsigned)((F + rows1 - 1) / rows1), (unsigned)P);
    const uint16_t* xb = (const uint16_t*)x;
    {
    dymoe_kernel_timer timer(ctx, DYMOE_K_GEMV_PHASE1, st);
    switch (nseg1) {
    case 1: hipLaunchKernelGGL((gemv_phase1_kernel<1>), g1, dim3(kGvThreads), 0, st, xb, idx, bits, table, H, F, E, k, rows1, hbuf); break;
    case 2: hipLaunchKernelGGL((gemv_phase1_kernel<2>), g1, dim3(kGvThreads), 0, st, xb, idx, bits, table, H, F, E, k, rows1, hbuf); break;
    case 3: hipLaunchKernelGGL((gemv_phase1_kernel<3>), g1, dim3(kGvThreads), 0, st, xb, idx, bits, table, H, F, E, k, rows1, hbuf); break;
    case 4: hipLaunchKernelGGL((gemv_phase1_kernel<4>), g1, dim3(kGvThreads), 0, st, xb, idx, bits, table, H, F, E, k, rows1, hbuf); break;
    default: return DYMOE_ENOTSUP;
    }
    }
    DYMOE_HIP_LAUNCH_CHECK();
    const dim3 g2((unsigned)((H + rows2 - 1) / rows2), (unsigned)nseg2, (unsigned)P);
    {
    dymoe_kernel_timer timer(ctx, DYMOE_K_GEMV_PHASE2, st);
    hipLaunchKernelGGL(gemv_phase2_kernel, g2, dim3(kGvThreads), 0, st, hbuf, idx, bits, table, H, F,
                       E, rows2, nseg2, part);
    }
    DYMOE_HIP_LAUNCH_CHECK();
    const long n = (long)T * H;
    dymoe_kernel_timer timer(ctx, DYMOE_K_GEMV_COMBINE, st);
    hipLaunchKernelGGL(gemv_combine_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, part,
                       idx, w, bits, T, H, E, k, nseg2, out_dtype, y);
    DYMOE_HIP_LAUNCH_CHECK();
    return DYMOE_OK;
}

}  // namespace dymoe
