// Internal helpers shared by the libdymoe HIP translation units (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>
#include <stdint.h>

#include "dymoe.h"

#include <vector>

// kernel ids of the per-kernel timing facility (dymoe_timing_*)
enum {
    DYMOE_K_ROUTE = 0,
    DYMOE_K_TOKEN_NORM,
    DYMOE_K_IMPORTANCE,
    DYMOE_K_ASSIGN,
    DYMOE_K_QUANTIZE,
    DYMOE_K_GEMV_PHASE1,
    DYMOE_K_GEMV_PHASE2,
    DYMOE_K_GEMV_COMBINE,
    DYMOE_K_PLAN,
    DYMOE_K_GEMM1,
    DYMOE_K_GEMM2,
    DYMOE_K_GEMM_COMBINE,
    DYMOE_K_STREAM_COPY,
    DYMOE_K_DECODE_FRONT,
    DYMOE_K_ATTN_STATS,
    DYMOE_K_ATTN_COLSUM,
    DYMOE_K_GPTQ_GROUP,
    DYMOE_K_GPTQ_TRAIL,
    DYMOE_K_GPTQ_HESSIAN,
    DYMOE_K_GPTQ_FACTOR,
    DYMOE_K_MFMA_PEAK,
    DYMOE_K_ROUTE_SELECT,
    DYMOE_K_COUNT
};

struct dymoe_timed_launch {
    int kernel;
    hipEvent_t start, stop;
};

struct dymoe_ctx {
    int device;
    int num_cu;
    void* static_scratch;                    // device address of this GPU's scratch array (dymoe_moe_ffn_mixed_noalloc)
    unsigned* device_flags;                  // device address of this GPU's condition word (dymoe_device_flags)
    unsigned timing_mask;                    // bit i set: time launches of kernel i
    std::vector<dymoe_timed_launch> timed;   // recorded, not yet read
};

// Launch a kernel.  When the context asks for this kernel to be timed, the
// launch carries a start and a stop event on the dispatch itself
// (hipExtLaunchKernelGGL), so the recorded interval is the kernel's own
// execution time on the launch stream, with no marker packets around it.
template <typename... KArgs, typename... Args>
inline void dymoe_launch(dymoe_ctx* ctx, int kernel_id, void (*kernel)(KArgs...), dim3 grid, dim3 block,
                         size_t smem, hipStream_t st, Args&&... args)
{
    if (ctx && ((ctx->timing_mask >> kernel_id) & 1u)) {
        dymoe_timed_launch rec;
        rec.kernel = kernel_id;
        if (hipEventCreate(&rec.start) == hipSuccess) {
            if (hipEventCreate(&rec.stop) == hipSuccess) {
                hipExtLaunchKernelGGL(kernel, grid, block, (uint32_t)smem, st, rec.start, rec.stop, 0,
                                      static_cast<KArgs>(args)...);
                ctx->timed.push_back(rec);
                return;
            }
            (void)hipEventDestroy(rec.start);
        }
    }
    hipLaunchKernelGGL(kernel, grid, block, (uint32_t)smem, st, static_cast<KArgs>(args)...);
}

#define DYMOE_REQUIRE(cond) \
    do {                    \
        if (!(cond)) return DYMOE_EINVAL; \
    } while (0)

#define DYMOE_HIP_LAUNCH_CHECK()                       \
    do {                                               \
        if (hipGetLastError() != hipSuccess) return DYMOE_EHIP; \
    } while (0)

static inline bool dymoe_aligned(const void* p, size_t a) { return ((uintptr_t)p % a) == 0; }

// Whether a table entry holds every pointer that running its expert at b bits reads: the three bf16 matrices for 16,
// codes, scales and zeros of the three matrices for 8 / 4 / 2.  The bit widths are chosen on the device, so the host
// cannot know which formats a launch will touch; the kernels ask this before the first access and leave out an
// expert whose selected format is absent (raising DYMOE_FLAG_FORMAT_MISSING) instead of reading through NULL.
// (Written out field by field: selecting one of the member arrays by a run-time index would force the entry into
// private memory.)
__host__ __device__ inline bool dymoe_fmt_present(const dymoe_expert_fmt& ex, int b)
{
    if (b == 16) return ex.w[0] && ex.w[1] && ex.w[2];
    if (b == 8)
        return ex.q8[0] && ex.q8[1] && ex.q8[2] && ex.s8[0] && ex.s8[1] && ex.s8[2] && ex.z8[0] && ex.z8[1] && ex.z8[2];
    if (b == 4)
        return ex.q4[0] && ex.q4[1] && ex.q4[2] && ex.s4[0] && ex.s4[1] && ex.s4[2] && ex.z4[0] && ex.z4[1] && ex.z4[2];
    if (b == 2)
        return ex.q2[0] && ex.q2[1] && ex.q2[2] && ex.s2[0] && ex.s2[1] && ex.s2[2] && ex.z2[0] && ex.z2[1] && ex.z2[2];
    return false;
}

namespace dymoe {

constexpr int kWave = 64;

typedef _Float16 half2_t __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
typedef _Float16 half8_t __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float float16_t __attribute__((ext_vector_type(16)));

// A pointer fetched from the expert table carries no address space, so a plain
// dereference becomes a flat instruction, which also occupies the LDS counter and
// makes every wait on LDS data wait on weight loads as well.  All table pointers
// are device memory: these helpers access them as such.
typedef uint32_t u32x2_t __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
#define DYMOE_GLOBAL __attribute__((address_space(1)))

// (HIP's uint2/uint4 are classes whose copy goes through a generic reference, so
// 8- and 16-byte values are moved as native vectors and converted afterwards.)
template <typename T>
__device__ __forceinline__ T load_global(const void* p)
{
    if constexpr (sizeof(T) == 16) {
        const u32x4_t v = *(const DYMOE_GLOBAL u32x4_t*)p;
        return __builtin_bit_cast(T, v);
    } else if constexpr (sizeof(T) == 8) {
        const u32x2_t v = *(const DYMOE_GLOBAL u32x2_t*)p;
        return __builtin_bit_cast(T, v);
    } else {
        return *(const DYMOE_GLOBAL T*)p;
    }
}
template <typename T>
__device__ __forceinline__ void store_global(void* p, T v)
{
    if constexpr (sizeof(T) == 16) *(DYMOE_GLOBAL u32x4_t*)p = __builtin_bit_cast(u32x4_t, v);
    else if constexpr (sizeof(T) == 8) *(DYMOE_GLOBAL u32x2_t*)p = __builtin_bit_cast(u32x2_t, v);
    else *(DYMOE_GLOBAL T*)p = v;
}

// The same load marked non-temporal: data streamed through once.
template <typename T>
__device__ __forceinline__ T load_global_nt(const void* p)
{
    if constexpr (sizeof(T) == 16) {
        const u32x4_t v = __builtin_nontemporal_load((const DYMOE_GLOBAL u32x4_t*)p);
        return __builtin_bit_cast(T, v);
    } else if constexpr (sizeof(T) == 8) {
        const u32x2_t v = __builtin_nontemporal_load((const DYMOE_GLOBAL u32x2_t*)p);
        return __builtin_bit_cast(T, v);
    } else {
        return __builtin_nontemporal_load((const DYMOE_GLOBAL T*)p);
    }
}

// The same store marked non-temporal: written once, not read again by this kernel.
template <typename T>
__device__ __forceinline__ void store_global_nt(void* p, T v)
{
    if constexpr (sizeof(T) == 16) __builtin_nontemporal_store(__builtin_bit_cast(u32x4_t, v), (DYMOE_GLOBAL u32x4_t*)p);
    else if constexpr (sizeof(T) == 8) __builtin_nontemporal_store(__builtin_bit_cast(u32x2_t, v), (DYMOE_GLOBAL u32x2_t*)p);
    else __builtin_nontemporal_store(v, (DYMOE_GLOBAL T*)p);
}

__device__ __forceinline__ float bf16_bits_to_f32(uint32_t b) { return __uint_as_float(b << 16); }
__device__ __forceinline__ float bf16_lo(uint32_t pair) { return __uint_as_float(pair << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t pair) { return __uint_as_float(pair & 0xffff0000u); }

// fp32 -> bf16 bits, round to nearest even (finite inputs)
__device__ __forceinline__ uint32_t f32_to_bf16_bits(float f)
{
    uint32_t u = __float_as_uint(f);
    return (u + 0x7fffu + ((u >> 16) & 1u)) >> 16;
}

__device__ __forceinline__ uint32_t f16_bits(_Float16 h) { return (uint32_t)__builtin_bit_cast(uint16_t, h); }
__device__ __forceinline__ _Float16 f16_from_bits(uint32_t b) { return __builtin_bit_cast(_Float16, (uint16_t)b); }

__device__ __forceinline__ uint32_t pack_half2(float lo, float hi)
{
    half2_t v = {(_Float16)lo, (_Float16)hi};
    return __builtin_bit_cast(uint32_t, v);
}

__device__ __forceinline__ float dot2_f16(uint32_t a, uint32_t b, float c)
{
    return __builtin_amdgcn_fdot2(__builtin_bit_cast(half2_t, a), __builtin_bit_cast(half2_t, b), c, false);
}

__device__ __forceinline__ float dot2_bf16(uint32_t a, uint32_t b, float c)
{
    return __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, a), __builtin_bit_cast(bf16x2_t, b), c, false);
}

__device__ __forceinline__ float wave_sum(float v)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, kWave);
    return v;
}

// Reductions over the 64 lanes through the data-parallel primitives (no LDS
// crossbar), returned in every lane.
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ float dpp_get(float v)
{
    // lanes whose row is masked out, or whose source lane does not exist, read 0
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, ROW_MASK, 0xF, true));
}

template <int CTRL, int ROW_MASK>
__device__ __forceinline__ float dpp_get_or_self(float v)
{
    // lanes whose row is masked out, or whose source lane does not exist, read their own value
    return __int_as_float(__builtin_amdgcn_update_dpp(__float_as_int(v), __float_as_int(v), CTRL, ROW_MASK, 0xF, false));
}

// (v & mask) | magic in one instruction.  With literal operands the compiler has
// to emit two (the three-operand form takes no literals), so the mask is handed
// over in a scalar register and the magic number in a vector register.
__device__ __forceinline__ uint32_t and_or(uint32_t v, uint32_t mask, uint32_t magic)
{
    uint32_t r;
    asm("v_and_or_b32 %0, %1, %2, %3" : "=v"(r) : "v"(v), "s"(mask), "v"(magic));
    return r;
}

__device__ __forceinline__ float wave_sum_dpp(float v)
{
    v += dpp_get<0xB1, 0xF>(v);    // quad_perm [1,0,3,2]
    v += dpp_get<0x4E, 0xF>(v);    // quad_perm [2,3,0,1]
    v += dpp_get<0x141, 0xF>(v);   // row_half_mirror
    v += dpp_get<0x140, 0xF>(v);   // row_mirror: every lane of a row holds the row's sum
    v += dpp_get<0x142, 0xA>(v);   // row_bcast15 into rows 1 and 3
    v += dpp_get<0x143, 0xC>(v);   // row_bcast31 into rows 2 and 3
    return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 63));
}

__device__ __forceinline__ int wave_sum_dpp_i32(int v)
{
    v += __builtin_amdgcn_update_dpp(0, v, 0xB1, 0xF, 0xF, true);
    v += __builtin_amdgcn_update_dpp(0, v, 0x4E, 0xF, 0xF, true);
    v += __builtin_amdgcn_update_dpp(0, v, 0x141, 0xF, 0xF, true);
    v += __builtin_amdgcn_update_dpp(0, v, 0x140, 0xF, 0xF, true);
    v += __builtin_amdgcn_update_dpp(0, v, 0x142, 0xA, 0xF, true);
    v += __builtin_amdgcn_update_dpp(0, v, 0x143, 0xC, 0xF, true);
    return __builtin_amdgcn_readlane(v, 63);
}

__device__ __forceinline__ float wave_max_dpp(float v)
{
    v = fmaxf(v, dpp_get_or_self<0xB1, 0xF>(v));
    v = fmaxf(v, dpp_get_or_self<0x4E, 0xF>(v));
    v = fmaxf(v, dpp_get_or_self<0x141, 0xF>(v));
    v = fmaxf(v, dpp_get_or_self<0x140, 0xF>(v));
    v = fmaxf(v, dpp_get_or_self<0x142, 0xA>(v));
    v = fmaxf(v, dpp_get_or_self<0x143, 0xC>(v));
    return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 63));
}

__device__ __forceinline__ float wave_max(float v)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, kWave));
    return v;
}

}  // namespace dymoe
