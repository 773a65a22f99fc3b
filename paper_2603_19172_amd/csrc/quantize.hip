// Group-wise asymmetric quantize-and-pack (bf16 -> int4 / int2 codes + fp16
// scale and zero per group of 64 columns).  Streaming, HBM-bound:
// every lane owns 8 consecutive bf16 (one 16-byte load), 8 lanes own a group.
//
// The arithmetic is an exact sequence of binary32 operations (this file is
// built with -ffp-contract=off): the codes must equal the reference's bit for
// bit, so nothing here may be fused, reassociated or approximated.
#include "common.hpp"

namespace dymoe {

constexpr int kQThreads = 256;
constexpr int kQUnroll = 4;  // 16-byte loads in flight per lane

template <int BITS>
__device__ __forceinline__ void quantize_chunk(const uint4 raw, long chunk,
                                               uint8_t* __restrict__ codes,
                                               uint16_t* __restrict__ scale,
                                               uint16_t* __restrict__ zero, int lane)
{
#pragma clang fp contract(off)
    constexpr int qmax = (1 << BITS) - 1;
    float v[8];
    v[0] = bf16_lo(raw.x); v[1] = bf16_hi(raw.x);
    v[2] = bf16_lo(raw.y); v[3] = bf16_hi(raw.y);
    v[4] = bf16_lo(raw.z); v[5] = bf16_hi(raw.z);
    v[6] = bf16_lo(raw.w); v[7] = bf16_hi(raw.w);
    float lo = v[0], hi = v[0];
#pragma unroll
    for (int i = 1; i < 8; i++) {
        lo = fminf(lo, v[i]);
        hi = fmaxf(hi, v[i]);
    }
    // the 8 lanes of a group are lane-aligned (chunks_per_row is a multiple of 8)
#pragma unroll
    for (int o = 1; o < 8; o <<= 1) {
        lo = fminf(lo, __shfl_xor(lo, o, kWave));
        hi = fmaxf(hi, __shfl_xor(hi, o, kWave));
    }
    const _Float16 zh = (_Float16)lo;                 // round to nearest even
    const float range = hi - lo;
    const float step = range / (float)qmax;           // correctly rounded division
    const _Float16 sh = (_Float16)step;
    const float m = (float)zh;
    const float s = (float)sh;
    const float inv = (s > 0.0f) ? (1.0f / s) : 0.0f;
    uint32_t word = 0;
#pragma unroll
    for (int i = 0; i < 8; i++) {
        const float d = v[i] - m;
        const float r = rintf(d * inv);
        int q = (int)r;
        q = q < 0 ? 0 : (q > qmax ? qmax : q);
        word |= (uint32_t)q << (BITS * i);
    }
    // rows are whole numbers of groups, so the flat chunk index addresses the
    // packed row-major outputs directly: 8 codes per chunk, 8 chunks per group
    if (BITS == 4) {
        *reinterpret_cast<uint32_t*>(codes + chunk * 4) = word;
    } else {
        // two lanes share one 32-bit store
        const uint32_t other = __shfl_down(word, 1, kWave);
        if ((lane & 1) == 0) *reinterpret_cast<uint32_t*>(codes + chunk * 2) = word | (other << 16);
    }
    if ((lane & 7) == 0) {
        scale[chunk >> 3] = (uint16_t)f16_bits(sh);
        zero[chunk >> 3] = (uint16_t)f16_bits(zh);
    }
}

template <int BITS>
__device__ __forceinline__ void quantize_block(const uint16_t* __restrict__ w, long n_chunks,
                                               uint8_t* __restrict__ codes,
                                               uint16_t* __restrict__ scale,
                                               uint16_t* __restrict__ zero, long block)
{
    const int lane = threadIdx.x & (kWave - 1);
    const long base = block * (long)(kQThreads * kQUnroll) + threadIdx.x;
    uint4 raw[kQUnroll];
#pragma unroll
    for (int u = 0; u < kQUnroll; u++) {
        const long c = base + (long)u * kQThreads;
        if (c < n_chunks) raw[u] = reinterpret_cast<const uint4*>(w)[c];
        else raw[u] = make_uint4(0, 0, 0, 0);
    }
#pragma unroll
    for (int u = 0; u < kQUnroll; u++) {
        const long c = base + (long)u * kQThreads;
        // n_chunks is a multiple of 8, so a group's 8 lanes are in or out together
        if (c < n_chunks) quantize_chunk<BITS>(raw[u], c, codes, scale, zero, lane);
    }
}

__global__ __launch_bounds__(kQThreads) void quantize_pack_kernel(
    const uint16_t* __restrict__ w, long n_chunks, int bits,
    uint8_t* __restrict__ codes, uint16_t* __restrict__ scale, uint16_t* __restrict__ zero)
{
    if (bits == 4) quantize_block<4>(w, n_chunks, codes, scale, zero, blockIdx.x);
    else quantize_block<2>(w, n_chunks, codes, scale, zero, blockIdx.x);
}

// One launch for a whole layer: blockIdx.y = 3*expert + matrix.  The expert's
// bit width is read on the device, so no decision goes through the host.
__global__ __launch_bounds__(kQThreads) void quantize_experts_kernel(
    const dymoe_expert_fmt* __restrict__ table, const uint8_t* __restrict__ bits,
    const int32_t* __restrict__ load, int H, int F)
{
    const int e = blockIdx.y / 3;
    const int mat = blockIdx.y - 3 * e;
    const int b = bits[e];
    if (b != 4 && b != 2) return;
    if (load != nullptr && load[e] <= 0) return;
    const long n_chunks = (long)H * (long)F / 8;
    const dymoe_expert_fmt ex = table[e];
    const uint16_t* w = reinterpret_cast<const uint16_t*>(ex.w[mat]);
    if (b == 4)
        quantize_block<4>(w, n_chunks, ex.q4[mat],
                          reinterpret_cast<uint16_t*>(ex.s4[mat]),
                          reinterpret_cast<uint16_t*>(ex.z4[mat]), blockIdx.x);
    else
        quantize_block<2>(w, n_chunks, ex.q2[mat],
                          reinterpret_cast<uint16_t*>(ex.s2[mat]),
                          reinterpret_cast<uint16_t*>(ex.z2[mat]), blockIdx.x);
}

}  // namespace dymoe

extern "C" {

int dymoe_quantize_pack(dymoe_ctx* ctx, const void* w, long N, long K, int bits, int group,
                        uint8_t* codes, void* scale, void* zero, void* stream)
{
    DYMOE_REQUIRE(N >= 0 && K > 0);
    DYMOE_REQUIRE(bits == 2 || bits == 4);
    DYMOE_REQUIRE(group > 0 && K % group == 0);
    if (N == 0) return (group != 64) ? DYMOE_ENOTSUP : (ctx ? DYMOE_OK : DYMOE_ENOCTX);  // nothing to read or write
    DYMOE_REQUIRE(w && codes && scale && zero);
    DYMOE_REQUIRE(dymoe_aligned(w, 16) && dymoe_aligned(codes, 4) && dymoe_aligned(scale, 2) &&
                  dymoe_aligned(zero, 2));
    if (group != 64) return DYMOE_ENOTSUP;
    if (!ctx) return DYMOE_ENOCTX;
    const long n_chunks = N * K / 8;
    const long per_block = dymoe::kQThreads * dymoe::kQUnroll;
    const long blocks = (n_chunks + per_block - 1) / per_block;
    if (blocks > 0x7fffffffL) return DYMOE_ENOTSUP;
    dymoe_kernel_timer timer(ctx, DYMOE_K_QUANTIZE, (hipStream_t)stream);
    hipLaunchKernelGGL(dymoe::quantize_pack_kernel, dim3((unsigned)blocks), dim3(dymoe::kQThreads), 0,
                       (hipStream_t)stream, (const uint16_t*)w, n_chunks, bits, codes,
                       (uint16_t*)scale, (uint16_t*)zero);
    DYMOE_HIP_LAUNCH_CHECK();
    return DYMOE_OK;
}

int dymoe_quantize_experts(dymoe_ctx* ctx, const dymoe_expert_fmt* table, const uint8_t* bits,
                           const int32_t* load, int E, int H, int F, int group, void* stream)
{
    DYMOE_REQUIRE(table && bits);
    DYMOE_REQUIRE(E > 0 && E <= DYMOE_MAX_EXPERTS && H > 0 && F > 0);
    DYMOE_REQUIRE(group > 0 && H % group == 0 && F % group == 0);
    if (group != 64) return DYMOE_ENOTSUP;
    if (!ctx) return DYMOE_ENOCTX;
    const long n_chunks = (long)H * (long)F / 8;
    const long per_block = dymoe::kQThreads * dymoe::kQUnroll;
    const long blocks = (n_chunks + per_block - 1) / per_block;
    if (blocks > 0x7fffffffL) return DYMOE_ENOTSUP;
    dymoe_kernel_timer timer(ctx, DYMOE_K_QUANTIZE, (hipStream_t)stream);
    hipLaunchKernelGGL(dymoe::quantize_experts_kernel, dim3((unsigned)blocks, (unsigned)(3 * E)),
                       dim3(dymoe::kQThreads), 0, (hipStream_t)stream, table, bits, load, H, F);
    DYMOE_HIP_LAUNCH_CHECK();
    return DYMOE_OK;
}

}  // extern "C"
