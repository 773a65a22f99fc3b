// Error-compensated quantize-and-pack (paper Sec. 5: GPTQ is the base quantizer
// of the paper's implementation).  Same outputs as the plain quantizer (codes,
// fp16 scale and zero per group of 64 columns, row-major), but a row is
// quantised column by column and what rounding takes away from column c is
// spread over the columns still to come, so that the layer's output on the
// calibration inputs changes least:
//     e = (v[c] - dequant(q_c)) / U[c,c],    v[j] = fma(-e, U[c,j], v[j])  for j > c,
// U the upper triangular factor of the inverse of the (damped) Hessian
// H = X^T X of the calibration inputs, H^-1 = U^T U.  Scale and zero of a group
// are taken from the row's corrected values when the group is reached.
//
// The arithmetic is an exact sequence of binary32 operations, columns in
// ascending order, one fused multiply-add per correction (this file is built
// with -ffp-contract=off, the fma is written out): the codes must equal the
// reference's bit for bit.  That fixes the structure: no matrix-core product
// for the trailing update (it would round differently), but the same work as
// a chain of fp32 FMAs in registers.
//
// Rows are independent, columns are not.  Per group of 64 columns two launches:
//   group kernel   a lane owns a row: the group's 64 values in registers, the
//                  64 x 64 diagonal block of U read through the scalar cache
//                  (every lane needs the same value); quantises the 64 columns
//                  in order, applies the corrections inside the group, writes
//                  codes, scale, zero and the 64 errors e of the row;
//   trail kernel   v[:, j] for all later columns j: 64 chained FMAs per element,
//                  a workgroup on a 64-row x 128-column tile with the errors and
//                  the 64 x 128 block of U in LDS, 8 x 4 elements per thread.
// The working copy v of the matrix (fp32) lives in the caller's workspace.
#include "common.hpp"

namespace dymoe {

constexpr int kGqGroup = 64;        // columns per group = columns per step
constexpr int kGqRows = 64;         // rows per workgroup in both kernels
constexpr int kGqTrailCols = 128;   // columns per workgroup of the trail kernel
constexpr int kGqTrailThreads = 256;

static inline size_t gq_round256(size_t v) { return (v + 255) & ~(size_t)255; }
static inline long gq_rows_padded(long N) { return (N + kGqRows - 1) / kGqRows * kGqRows; }

__global__ __launch_bounds__(256) void gptq_widen_kernel(const uint16_t* __restrict__ w, long n_elems,
                                                         float* __restrict__ v)
{
    const long i = ((long)blockIdx.x * 256 + threadIdx.x) * 8;
    if (i >= n_elems) return;                       // n_elems is a multiple of 64
    const uint4 raw = load_global<uint4>(w + i);
    float4 a, b;
    a.x = bf16_lo(raw.x); a.y = bf16_hi(raw.x); a.z = bf16_lo(raw.y); a.w = bf16_hi(raw.y);
    b.x = bf16_lo(raw.z); b.y = bf16_hi(raw.z); b.z = bf16_lo(raw.w); b.w = bf16_hi(raw.w);
    *reinterpret_cast<float4*>(v + i) = a;
    *reinterpret_cast<float4*>(v + i + 4) = b;
}

// err [64][n_pad]: e of column base + c for row r at err[c * n_pad + r].
template <int BITS>
__global__ __launch_bounds__(kGqRows) void gptq_group_kernel(
    const float* __restrict__ v, const float* __restrict__ u, long N, long K, long base, long n_pad,
    uint8_t* __restrict__ codes, uint16_t* __restrict__ scale, uint16_t* __restrict__ zero,
    float* __restrict__ err)
{
#pragma clang fp contract(off)
    constexpr int qmax = (1 << BITS) - 1;
    constexpr int per_word = 32 / BITS;
    constexpr int n_words = kGqGroup / per_word;    // 16 (int8), 8 (int4), 4 (int2)
    const long slot = (long)blockIdx.x * kGqRows + threadIdx.x;   // < n_pad
    const long row = min(slot, N - 1);              // lanes past the last row redo it and store nothing but their errors
    float x[kGqGroup];
#pragma unroll
    for (int c = 0; c < kGqGroup / 4; c++) {
        const float4 q = *reinterpret_cast<const float4*>(v + row * K + base + 4 * c);
        x[4 * c + 0] = q.x; x[4 * c + 1] = q.y; x[4 * c + 2] = q.z; x[4 * c + 3] = q.w;
    }
    float lo = x[0], hi = x[0];
#pragma unroll
    for (int i = 1; i < kGqGroup; i++) {
        lo = fminf(lo, x[i]);
        hi = fmaxf(hi, x[i]);
    }
    const _Float16 zh = (_Float16)lo;               // round to nearest even
    const float range = hi - lo;
    const float step = range / (float)qmax;         // correctly rounded division
    const _Float16 sh = (_Float16)step;
    const float m = (float)zh;
    const float s = (float)sh;
    const float inv = (s > 0.0f) ? (1.0f / s) : 0.0f;
    const float* __restrict__ ub = u + base * K + base;      // the diagonal block: the same address in every lane
    uint32_t words[n_words];
#pragma unroll
    for (int i = 0; i < n_words; i++) words[i] = 0u;
#pragma unroll
    for (int i = 0; i < kGqGroup; i++) {
        const float d = x[i] - m;
        float r = __builtin_rintf(d * inv);
        r = fminf(fmaxf(r, 0.0f), (float)qmax);
        words[i / per_word] |= (uint32_t)(int)r << (BITS * (i % per_word));
        float dq = r * s;
        dq = dq + m;
        const float e = (x[i] - dq) / ub[(long)i * K + i];
        err[(long)i * n_pad + slot] = e;
        const float ne = -e;
#pragma unroll
        for (int j = i + 1; j < kGqGroup; j++) x[j] = __builtin_fmaf(ne, ub[(long)i * K + j], x[j]);
    }
    if (slot < N) {
        const long G = K / kGqGroup;
        uint8_t* dst = codes + row * (K * BITS / 8) + base * BITS / 8;
#pragma unroll
        for (int i = 0; i < n_words / 4; i++)
            store_global(dst + 16 * i, make_uint4(words[4 * i], words[4 * i + 1], words[4 * i + 2], words[4 * i + 3]));
        store_global(scale + row * G + base / kGqGroup, (uint16_t)f16_bits(sh));
        store_global(zero + row * G + base / kGqGroup, (uint16_t)f16_bits(zh));
    }
}

// v[r, j] = fma(-err[c][r], U[base + c, j], v[r, j]) for c = 0 .. 63 in order, all j >= base + 64.
__global__ __launch_bounds__(kGqTrailThreads) void gptq_trail_kernel(
    float* __restrict__ v, const float* __restrict__ u, const float* __restrict__ err, long N, long K,
    long base, long n_pad)
{
    __shared__ __attribute__((aligned(16))) float s_e[kGqGroup][kGqRows];
    __shared__ __attribute__((aligned(16))) float s_u[kGqGroup][kGqTrailCols];
    const int tid = threadIdx.x;
    const long col0 = base + kGqGroup + (long)blockIdx.x * kGqTrailCols;
    const long row0 = (long)blockIdx.y * kGqRows;
#pragma unroll
    for (int i = 0; i < kGqGroup * kGqRows / 4 / kGqTrailThreads; i++) {
        const int at = (i * kGqTrailThreads + tid) * 4;
        const int c = at / kGqRows, r = at % kGqRows;
        *reinterpret_cast<float4*>(&s_e[c][r]) = *reinterpret_cast<const float4*>(err + (long)c * n_pad + row0 + r);
    }
#pragma unroll
    for (int i = 0; i < kGqGroup * kGqTrailCols / 4 / kGqTrailThreads; i++) {
        const int at = (i * kGqTrailThreads + tid) * 4;
        const int c = at / kGqTrailCols, n = at % kGqTrailCols;
        float4 q = make_float4(0.f, 0.f, 0.f, 0.f);
        if (col0 + n < K) q = *reinterpret_cast<const float4*>(u + (base + c) * K + col0 + n);
        *reinterpret_cast<float4*>(&s_u[c][n]) = q;
    }
    __syncthreads();
    const int tx = tid & 31, ty = tid >> 5;
    const long col = col0 + 4 * tx;
    const long row = row0 + 8 * ty;
    if (col >= K) return;
    float4 acc[8];
#pragma unroll
    for (int i = 0; i < 8; i++) {
        acc[i] = make_float4(0.f, 0.f, 0.f, 0.f);
        if (row + i < N) acc[i] = *reinterpret_cast<const float4*>(v + (row + i) * K + col);
    }
#pragma unroll 4
    for (int c = 0; c < kGqGroup; c++) {
        const float4 e0 = *reinterpret_cast<const float4*>(&s_e[c][8 * ty]);
        const float4 e1 = *reinterpret_cast<const float4*>(&s_e[c][8 * ty + 4]);
        const float4 uu = *reinterpret_cast<const float4*>(&s_u[c][4 * tx]);
        const float ne[8] = {-e0.x, -e0.y, -e0.z, -e0.w, -e1.x, -e1.y, -e1.z, -e1.w};
#pragma unroll
        for (int i = 0; i < 8; i++) {
            acc[i].x = __builtin_fmaf(ne[i], uu.x, acc[i].x);
            acc[i].y = __builtin_fmaf(ne[i], uu.y, acc[i].y);
            acc[i].z = __builtin_fmaf(ne[i], uu.z, acc[i].z);
            acc[i].w = __builtin_fmaf(ne[i], uu.w, acc[i].w);
        }
    }
#pragma unroll
    for (int i = 0; i < 8; i++)
        if (row + i < N) *reinterpret_cast<float4*>(v + (row + i) * K + col) = acc[i];
}

}  // namespace dymoe

extern "C" {

size_t dymoe_gptq_workspace_bytes(long N, long K)
{
    if (N <= 0 || K <= 0) return 0;
    return dymoe::gq_round256((size_t)N * (size_t)K * 4) +
           dymoe::gq_round256((size_t)dymoe::kGqGroup * (size_t)dymoe::gq_rows_padded(N) * 4);
}

int dymoe_gptq_quantize_pack(dymoe_ctx* ctx, const void* w_bf16, const float* u, long N, long K, int bits, int group,
                             uint8_t* codes, void* scale, void* zero, void* workspace, size_t workspace_bytes,
                             void* stream)
{
    using namespace dymoe;
    DYMOE_REQUIRE(w_bf16 && u && codes && scale && zero && workspace);
    DYMOE_REQUIRE(N > 0 && K > 0 && (bits == 2 || bits == 4 || bits == 8));
    DYMOE_REQUIRE(group == kGqGroup && K % kGqGroup == 0);
    DYMOE_REQUIRE(N * K < ((long)1 << 40));
    DYMOE_REQUIRE(dymoe_aligned(w_bf16, 16) && dymoe_aligned(u, 16) && dymoe_aligned(codes, 16) &&
                  dymoe_aligned(scale, 2) && dymoe_aligned(zero, 2) && dymoe_aligned(workspace, 256));
    if (workspace_bytes < dymoe_gptq_workspace_bytes(N, K)) return DYMOE_ENOSPC;
    if (!ctx) return DYMOE_ENOCTX;
    hipStream_t st = (hipStream_t)stream;
    const long n_pad = gq_rows_padded(N);
    float* v = reinterpret_cast<float*>(workspace);
    float* err = reinterpret_cast<float*>((char*)workspace + gq_round256((size_t)N * (size_t)K * 4));
    const long n_elems = N * K;
    hipLaunchKernelGGL(gptq_widen_kernel, dim3((unsigned)((n_elems / 8 + 255) / 256)), dim3(256), 0, st,
                       (const uint16_t*)w_bf16, n_elems, v);
    DYMOE_HIP_LAUNCH_CHECK();
    const dim3 grid_a((unsigned)(n_pad / kGqRows));
    for (long base = 0; base < K; base += kGqGroup) {
        switch (bits) {
        case 8:
            dymoe_launch(ctx, DYMOE_K_GPTQ_GROUP, gptq_group_kernel<8>, grid_a, dim3(kGqRows), 0, st, (const float*)v, u,
                         N, K, base, n_pad, codes, (uint16_t*)scale, (uint16_t*)zero, err);
            break;
        case 4:
            dymoe_launch(ctx, DYMOE_K_GPTQ_GROUP, gptq_group_kernel<4>, grid_a, dim3(kGqRows), 0, st, (const float*)v, u,
                         N, K, base, n_pad, codes, (uint16_t*)scale, (uint16_t*)zero, err);
            break;
        default:
            dymoe_launch(ctx, DYMOE_K_GPTQ_GROUP, gptq_group_kernel<2>, grid_a, dim3(kGqRows), 0, st, (const float*)v, u,
                         N, K, base, n_pad, codes, (uint16_t*)scale, (uint16_t*)zero, err);
            break;
        }
        DYMOE_HIP_LAUNCH_CHECK();
        const long rest = K - base - kGqGroup;
        if (rest > 0) {
            const dim3 grid_b((unsigned)((rest + kGqTrailCols - 1) / kGqTrailCols), (unsigned)(n_pad / kGqRows));
            dymoe_launch(ctx, DYMOE_K_GPTQ_TRAIL, gptq_trail_kernel, grid_b, dim3(kGqTrailThreads), 0, st, v, u,
                         (const float*)err, N, K, base, n_pad);
            DYMOE_HIP_LAUNCH_CHECK();
        }
    }
    return DYMOE_OK;
}

}  // extern "C"
