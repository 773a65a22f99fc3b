// dymoe_moe_ffn_mixed: argument checks and the choice between the decode
// (GEMV) and prefill (grouped GEMM) paths.
#include "common.hpp"
#include "assign.hpp"
#include "ffn_layout.hpp"

// Scratch of the entry point that allocates nothing.  One copy per GPU the library runs on, held until the
// process ends; every call on a GPU shares that GPU's copy.  In host code the array's name is only a stand-in: the
// device address comes from hipGetSymbolAddress (ffn_static_scratch_address) and is what every launch is given.
static __device__ __align__(256) unsigned char scratch[DYMOE_STATIC_SCRATCH_BYTES];

// Conditions the kernels met and went on from (DYMOE_FLAG_*), one word per GPU; read and cleared by
// dymoe_device_flags.  Handled like the scratch array: launches are given the address, never the name.
static __device__ unsigned device_flags;

namespace dymoe {
// Device address of this GPU's scratch array; the device must be current.
int ffn_static_scratch_address(void** out)
{
    void* p = nullptr;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || p == nullptr) return DYMOE_EHIP;
    *out = p;
    return DYMOE_OK;
}

// Device address of this GPU's condition word; the device must be current.
int ffn_device_flags_address(unsigned** out)
{
    void* p = nullptr;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(device_flags)) != hipSuccess || p == nullptr) return DYMOE_EHIP;
    *out = static_cast<unsigned*>(p);
    return DYMOE_OK;
}

int ffn_gemv_launch(dymoe_ctx* ctx, const void* x, const int32_t* idx, const float* w, const uint8_t* bits,
                    const dymoe_expert_fmt* table, int T, int H, int F, int E, int k,
                    int out_dtype, void* y, void* workspace, hipStream_t st);
int ffn_gemm_launch(dymoe_ctx* ctx, const void* x, const int32_t* idx, const float* w, const uint8_t* bits,
                    const dymoe_expert_fmt* table, int T, int H, int F, int E, int k,
                    int out_dtype, void* y, void* workspace, hipStream_t st);
bool ffn_gemm_fits(int T, int H, int F, int E, int k);
bool decode_fused_fits(int T, int H, int E, int k);
int decode_fused_launch(dymoe_ctx* ctx, const void* x, const void* wg, const float* bias, const TierTable& tt,
                        int floor_bits, const dymoe_expert_fmt* table, int T, int H, int F, int E, int k, int renorm,
                        int out_dtype, int32_t* idx, float* w, float* probs, float* importance, int32_t* load,
                        uint8_t* bits, int32_t* rank, void* y, void* workspace, hipStream_t st);
}  // namespace dymoe

// Argument checks shared by the two entry points; on DYMOE_OK *path holds the path that will run.
static int ffn_check(const void* x, const int32_t* idx, const float* w, const uint8_t* bits,
                     const dymoe_expert_fmt* table, int T, int H, int F, int E, int k, int group, int out_dtype,
                     int* path, const void* y, const void* workspace, size_t workspace_bytes)
{
    DYMOE_REQUIRE(T >= 0 && H > 0 && F > 0 && E > 0 && k > 0 && k <= E);
    DYMOE_REQUIRE(bits && table && workspace);
    if (T > 0) DYMOE_REQUIRE(x && idx && w && y);  // empty step: nothing to read or write
    DYMOE_REQUIRE(group > 0 && H % group == 0 && F % group == 0);
    DYMOE_REQUIRE(out_dtype == DYMOE_OUT_BF16 || out_dtype == DYMOE_OUT_F32);
    DYMOE_REQUIRE(*path == DYMOE_PATH_AUTO || *path == DYMOE_PATH_GEMV || *path == DYMOE_PATH_GEMM);
    DYMOE_REQUIRE(dymoe_aligned(x, 16) && dymoe_aligned(y, 16) && dymoe_aligned(workspace, 256));
    if (group != 64 || E > DYMOE_MAX_EXPERTS) return DYMOE_ENOTSUP;
    if ((long)T * k > 0x7fffffffL / 4) return DYMOE_ENOTSUP;
    if (workspace_bytes < dymoe::ffn_layout(T, H, F, E, k).total) return DYMOE_ENOSPC;
    const bool gemm_ok = (H % 128 == 0) && (F % 128 == 0);
    const bool gemv_ok = (H <= 4 * dymoe::kSeg) && ((long)T * k <= 65535);
    if (*path == DYMOE_PATH_AUTO) *path = (T <= 4 || !gemm_ok) ? DYMOE_PATH_GEMV : DYMOE_PATH_GEMM;
    if (*path == DYMOE_PATH_GEMV && !gemv_ok) return DYMOE_ENOTSUP;
    if (*path == DYMOE_PATH_GEMM && !gemm_ok) return DYMOE_ENOTSUP;
    if (*path == DYMOE_PATH_GEMM && !dymoe::ffn_gemm_fits(T, H, F, E, k)) return DYMOE_ENOTSUP;
    return DYMOE_OK;
}

extern "C" int dymoe_moe_ffn_mixed(dymoe_ctx* ctx, const void* x, const int32_t* idx,
                                   const float* w, const uint8_t* bits,
                                   const dymoe_expert_fmt* table, int T, int H, int F, int E,
                                   int k, int group, int out_dtype, int path, void* y,
                                   void* workspace, size_t workspace_bytes, void* stream)
{
    const int rc = ffn_check(x, idx, w, bits, table, T, H, F, E, k, group, out_dtype, &path, y, workspace, workspace_bytes);
    if (rc != DYMOE_OK) return rc;
    if (!ctx) return DYMOE_ENOCTX;
    if (T == 0) return DYMOE_OK;
    if (path == DYMOE_PATH_GEMV)
        return dymoe::ffn_gemv_launch(ctx, x, idx, w, bits, table, T, H, F, E, k, out_dtype, y, workspace,
                                      (hipStream_t)stream);
    return dymoe::ffn_gemm_launch(ctx, x, idx, w, bits, table, T, H, F, E, k, out_dtype, y, workspace,
                                  (hipStream_t)stream);
}

extern "C" int dymoe_moe_ffn_mixed_noalloc(dymoe_ctx* ctx, const void* x, const int32_t* idx,
                                           const float* w, const uint8_t* bits,
                                           const dymoe_expert_fmt* table, int T, int H, int F, int E,
                                           int k, int group, int out_dtype, int path, void* y, void* stream)
{
    // sizes are judged against the fixed capacity; the address stands in for the pointer checks until a context is there
    void* ws = ctx ? ctx->static_scratch : reinterpret_cast<void*>((uintptr_t)256);
    const int rc = ffn_check(x, idx, w, bits, table, T, H, F, E, k, group, out_dtype, &path, y, ws,
                             (size_t)DYMOE_STATIC_SCRATCH_BYTES);
    if (rc != DYMOE_OK) return rc;
    if (!ctx) return DYMOE_ENOCTX;
    if (!ctx->static_scratch) return DYMOE_EHIP;
    if (T == 0) return DYMOE_OK;
    // per-kernel timing creates events; this entry point creates nothing
    const unsigned mask = ctx->timing_mask;
    ctx->timing_mask = 0;
    const int out = (path == DYMOE_PATH_GEMV)
        ? dymoe::ffn_gemv_launch(ctx, x, idx, w, bits, table, T, H, F, E, k, out_dtype, y, ws, (hipStream_t)stream)
        : dymoe::ffn_gemm_launch(ctx, x, idx, w, bits, table, T, H, F, E, k, out_dtype, y, ws, (hipStream_t)stream);
    ctx->timing_mask = mask;
    return out;
}

extern "C" int dymoe_decode_step(dymoe_ctx* ctx, const void* x, const void* wg, const float* bias, int T, int H, int F,
                                 int E, int k, int renorm, int n_tiers, const int32_t* tier_count,
                                 const uint8_t* tier_bits, int floor_bits, const dymoe_expert_fmt* table, int group,
                                 int out_dtype, int32_t* idx, float* w, float* probs, float* importance,
                                 int32_t* load, uint8_t* bits, int32_t* rank, void* y, void* workspace,
                                 size_t workspace_bytes, void* stream)
{
    // the front end's checks, then the FFN's
    DYMOE_REQUIRE(T >= 1 && H > 0 && F > 0 && E > 0 && k > 0 && k <= E && H % 8 == 0);
    DYMOE_REQUIRE(x && wg && idx && w && importance && load && bits);
    DYMOE_REQUIRE(dymoe_aligned(x, 16) && dymoe_aligned(wg, 16));
    DYMOE_REQUIRE(floor_bits == 0 || floor_bits == 2 || floor_bits == 4 || floor_bits == 8 || floor_bits == 16);
    dymoe::TierTable tt;
    DYMOE_REQUIRE(dymoe::make_tier_table(E, n_tiers, tier_count, tier_bits, tt) == DYMOE_OK);
    int path = DYMOE_PATH_GEMV;
    const int rc = ffn_check(x, idx, w, bits, table, T, H, F, E, k, group, out_dtype, &path, y, workspace, workspace_bytes);
    if (rc != DYMOE_OK) return rc;
    if (!dymoe::decode_fused_fits(T, H, E, k)) return DYMOE_ENOTSUP;
    if (!ctx) return DYMOE_ENOCTX;
    return dymoe::decode_fused_launch(ctx, x, wg, bias, tt, floor_bits, table, T, H, F, E, k, renorm, out_dtype, idx, w,
                                      probs, importance, load, bits, rank, y, workspace, (hipStream_t)stream);
}
