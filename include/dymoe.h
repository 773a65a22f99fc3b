/*
 * libdymoe: one Mixture-of-Experts layer under dynamic mixed precision
 * (DyMoE), hand-written HIP for AMD gfx950, behind a plain C ABI.
 *
 * Pipeline of one layer (paper Sec. 4.1, steps 1-4 of the system overview):
 *   dymoe_route_topk        router gating and top-k
 *   dymoe_expert_importance per-expert importance (prefill: heavy-hitter token
 *                           load; decode: gate score)
 *   dymoe_assign_precision  importance- and depth-based bit-width per expert
 *   dymoe_quantize_pack /   group-wise quantize-and-pack of expert weights
 *   dymoe_quantize_experts
 *   dymoe_moe_ffn_mixed     dequant-fused SwiGLU expert FFN over experts of
 *                           differing precisions
 *
 * Conventions that hold for every call unless a comment says otherwise:
 *  - Every pointer is a DEVICE pointer; arguments marked "host" are host
 *    pointers that are read before the call returns.
 *  - The caller allocates and owns every buffer.  The library never allocates
 *    or frees device memory and keeps no pointer after the call returns
 *    (dymoe_prefetch_submit creates an event that the caller releases).
 *  - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *    Calls enqueue work and return without synchronising; nothing is read
 *    back to the host, so the five steps chain on one stream with no host
 *    round trip.
 *  - bf16 and fp16 tensors are raw 16-bit patterns.  Matrices are row-major
 *    with the contraction ("in") dimension contiguous: W1, W3 are [F,H],
 *    W2 is [H,F], the router weight is [E,H].
 *  - Return value: 0 on success, a negative DYMOE_E* code otherwise.
 *    Arguments are validated before any GPU work is issued; a failing call
 *    has enqueued nothing.  A tensor with zero rows (T = 0, N = 0) may be
 *    passed as NULL; such a call is a successful no-op.
 */
#ifndef DYMOE_H
#define DYMOE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define DYMOE_OK 0
#define DYMOE_EINVAL (-1)  /* bad argument: null pointer, bad size, bad bit width, misaligned */
#define DYMOE_ENOSPC (-2)  /* workspace too small */
#define DYMOE_EHIP (-3)    /* a HIP runtime call failed */
#define DYMOE_ENOTSUP (-4) /* valid in principle, outside what the kernels cover */
#define DYMOE_ENOCTX (-5)  /* context is NULL (checked after the other arguments) */

/* bits of the per-device condition word (dymoe_device_flags) */
#define DYMOE_FLAG_FORMAT_MISSING 1u /* an expert with tokens was assigned a precision its table entry does not hold */

#define DYMOE_PHASE_PREFILL 0
#define DYMOE_PHASE_DECODE 1

/* out_dtype of dymoe_moe_ffn_mixed */
#define DYMOE_OUT_BF16 0
#define DYMOE_OUT_F32 1

/* path of dymoe_moe_ffn_mixed */
#define DYMOE_PATH_AUTO 0
#define DYMOE_PATH_GEMV 1  /* bandwidth-bound dequant GEMV per (token, expert) pair */
#define DYMOE_PATH_GEMM 2  /* tokens grouped by expert, MFMA grouped GEMM */

/* layout of packed expert weights (codes + scale/zero, and the bf16 tile copy) */
#define DYMOE_LAYOUT_ROWMAJOR 0 /* as dymoe_quantize_pack writes: what the GEMV path reads */
#define DYMOE_LAYOUT_TILE 1     /* 32-row x 128-column tiles: what the GEMM path reads */

#define DYMOE_MAX_TIERS 8
#define DYMOE_FRONT_MAX_TOKENS 16   /* tokens per step of dymoe_decode_front */
#define DYMOE_MAX_EXPERTS 1024

/* opaque; holds the device ordinal, its properties and the records of the
 * per-kernel timing facility.  It owns no device memory.  Calls that share a
 * context must come from one host thread at a time. */
typedef struct dymoe_ctx dymoe_ctx;

/*
 * One expert's weights in every precision the caller has materialised.
 * Index 0, 1, 2 of each array = W1 (gate, [F,H]), W3 (up, [F,H]), W2 (down, [H,F]).
 * w: bf16, row-major.  q8/q4/q2: packed codes; s8, z8, s4, z4, s2, z2: fp16 scale
 * and zero, one per group of 64 columns (the 8-bit state is the top of the
 * paper's precision spectrum, Sec. 1).  wt: optional copy of w in the tile layout
 * (dymoe_pack_tiles), read by the GEMM path for 16-bit experts; when NULL that
 * path reads w row by row (slower).
 * Entries for precisions that are never selected may be NULL.  The precisions are
 * chosen on the device, so no host check can know which entries a launch will read:
 * dymoe_moe_ffn_mixed, dymoe_decode_step and dymoe_quantize_experts test the pointers
 * of the selected format (for 16 bits w, for 8 / 4 / 2 the codes, scales and zeros,
 * of all three matrices; for the quantiser also its source w) before the first
 * access, leave the expert out as if it had been assigned 0 bits when one is NULL
 * (the quantiser writes nothing for it), and raise DYMOE_FLAG_FORMAT_MISSING in the
 * device's condition word (dymoe_device_flags).  A non-NULL pointer is trusted.
 * The table lives in device memory ([E] of these).
 *
 * Two layouts of a packed [N,K] matrix exist, with the same bytes in a
 * different order (N multiple of 32 and K multiple of 128 for the tile one):
 *  DYMOE_LAYOUT_ROWMAJOR  codes [N, K*bits/8], scale and zero [N, K/64].
 *  DYMOE_LAYOUT_TILE      tiles of 32 rows x 128 columns, tile (nt, kt) at index
 *    nt*(K/128)+kt.  "Lane" l = 32*kb + r of a tile owns row 32*nt+r, columns
 *    128*kt+64*kb .. +64 (one quantisation group).  bf16: 8 KiB per tile, the
 *    lane's chunk j (8 columns, 16 bytes) at byte j*1024 + l*16.  int4: 2 KiB
 *    of codes per tile, the lane's chunk c (32 codes) at byte c*1024 + l*16.
 *    int2: 1 KiB per tile, the lane's 64 codes at byte l*16.  int8: 4 KiB per
 *    tile, the lane's chunk c (16 codes) at byte c*1024 + l*16.  Codes inside a
 *    chunk are packed as in the row-major layout.  scale / zero: 64 fp16 per
 *    tile, the lane's at index l.
 * The GEMV path of dymoe_moe_ffn_mixed reads the codes row-major, the GEMM path
 * reads them tiled: quantize with the layout of the path that will run.
 * (q8/s8/z8 were added after the other fields and sit at the end.)
 */
typedef struct {
    const void* w[3];
    const void* wt[3];
    uint8_t* q4[3];
    void* s4[3];
    void* z4[3];
    uint8_t* q2[3];
    void* s2[3];
    void* z2[3];
    uint8_t* q8[3];
    void* s8[3];
    void* z8[3];
} dymoe_expert_fmt;

/* Create / destroy a context bound to HIP device `device`.  Host calls. */
int dymoe_create(dymoe_ctx** out, int device);
void dymoe_destroy(dymoe_ctx* ctx);

/*
 * Conditions the kernels met and went on from since the last call of this function
 * on the context's device (DYMOE_FLAG_*): waits for `stream`, copies the device's
 * condition word to *flags and clears it when it was not zero.  One word per device
 * and process, shared by every context on that device.  A host call that
 * synchronises: not for use during stream capture, and not needed on the hot path
 * (a caller whose tables hold every format its tiers and floors can name never
 * sees a bit set).  Errors: DYMOE_EINVAL (flags NULL), DYMOE_ENOCTX, DYMOE_EHIP.
 */
int dymoe_device_flags(dymoe_ctx* ctx, unsigned* flags, void* stream);

/*
 * The test the kernels apply to a table entry before running its expert at `bits`
 * (see dymoe_expert_fmt), on a HOST copy of the entry: 1 when every pointer of that
 * format is non-NULL, 0 otherwise (also for a NULL entry or a bit width other than
 * 16, 8, 4, 2).  Pure host function; lets a caller check a table against the
 * precisions its tiers and floors can name before uploading it.
 */
int dymoe_format_present(const dymoe_expert_fmt* entry, int bits);

/* Static, human-readable text of an error code. */
const char* dymoe_strerror(int code);

/* Bytes of workspace dymoe_moe_ffn_mixed needs for these sizes (either path).
 * Pure host function; returns 0 for invalid sizes. */
size_t dymoe_workspace_bytes(int T, int H, int F, int E, int k);

/*
 * Router gating and top-k (paper Sec. 2.1; gate form of Sec. 4.4.1:
 * g = Softmax(h W_g), selection = TopK_k(g)).
 *   logit[t,e] = sum_h x[t,h] * wg[e,h] (+ bias[e]),  fp32 accumulation
 *   probs[t,:] = softmax over all E experts
 *   idx[t,0..k) = the k experts with the largest logit, descending, ties to
 *                 the lower index;  w[t,j] = probs[t, idx[t,j]], divided by
 *                 their sum when renorm != 0.
 * x [T,H] bf16, wg [E,H] bf16, bias [E] fp32 or NULL,
 * idx [T,k] int32, w [T,k] fp32, probs [T,E] fp32 or NULL.
 * Limits: 1 <= k <= E <= DYMOE_MAX_EXPERTS, H multiple of 8, H <= 16384.
 * One or two kernel launches on `stream`, by size; with two, probs holds the
 * logits between them (its contents are undefined until the call's work is done,
 * as for any output).
 */
int dymoe_route_topk(dymoe_ctx* ctx, const void* x, const void* wg, const float* bias,
                     int T, int H, int E, int k, int renorm,
                     int32_t* idx, float* w, float* probs, void* stream);

/*
 * Activation-norm token score s_t = ||x_t||_2 (fp32).  Stand-in for the
 * attention-derived token importance of paper Sec. 4.2.1 (first equation)
 * where no attention block is at hand (see dymoe_token_score_attention).
 * x [T,H] bf16, score [T] fp32.  H multiple of 8.
 */
int dymoe_token_score_norm(dymoe_ctx* ctx, const void* x, int T, int H, float* score,
                           void* stream);

/*
 * Attention-derived token score (paper Sec. 4.2.1, first equation):
 *   s_i = (1/n_heads) sum_h a_i^(h),
 * with a_i^(h) read as the attention token i RECEIVES in head h, averaged over
 * the T queries: a_i^(h) = (1/T) sum_q P^(h)[q,i], P^(h) = softmax over keys of
 * (q_q . k_i) * scale; causal = 1 masks the keys after the query.  The scores
 * sum to 1.  Feed `score` to dymoe_expert_importance as token_score.
 * q [T, n_heads, head_dim] bf16, k [T, n_kv_heads, head_dim] bf16 (token-major,
 * as a fused QKV projection writes them), 16-byte aligned; query head h reads
 * key head h / (n_heads / n_kv_heads).  scale > 0, or 0 for 1/sqrt(head_dim).
 * score [T] fp32.  workspace: device, 256-byte aligned, at least
 * dymoe_attention_workspace_bytes(T, n_heads) bytes (softmax statistics and
 * per-head sums); owned by the caller, free for reuse when the call's work on
 * `stream` has completed.  Deterministic (no atomics).
 * Limits: head_dim 64 or 128 (others: DYMOE_ENOTSUP); n_heads multiple of
 * n_kv_heads.  T = 0: nothing is read or written.
 */
size_t dymoe_attention_workspace_bytes(int T, int n_heads);
int dymoe_token_score_attention(dymoe_ctx* ctx, const void* q, const void* k, int T, int n_heads,
                                int n_kv_heads, int head_dim, float scale, int causal, float* score,
                                void* workspace, size_t workspace_bytes, void* stream);

/*
 * Per-expert importance (paper Sec. 4.2).
 * phase = DYMOE_PHASE_PREFILL (Sec. 4.2.1): T_imp = the k_hh tokens with the
 *   largest token_score (ties to the lower token index);
 *   importance[e] (int32) = number of (token, slot) pairs with token in T_imp and
 *   idx[token,slot] = e;  load[e] (int32) = that count over all tokens (also the
 *   token-frequency count of Sec. 4.4.1).  token_score [T] fp32 is required,
 *   probs is ignored.
 * phase = DYMOE_PHASE_DECODE (Sec. 4.2.2): importance[e] (fp32) = probs[0,e],
 *   the gating score; for T > 1 the mean over the T tokens.  load as above.
 *   probs [T,E] fp32 is required, token_score and k_hh are ignored.
 * idx [T,k] int32 with values in [0,E); entries outside that range are skipped.
 * importance [E] (4 bytes per entry, type by phase), load [E] int32.
 */
int dymoe_expert_importance(dymoe_ctx* ctx, int phase, const int32_t* idx, const float* probs,
                            const float* token_score, int T, int E, int k, int k_hh,
                            void* importance, int32_t* load, void* stream);

/*
 * Depth-aware retention schedule (paper Sec. 4.3), pure host function:
 *   r(l) = (1 - lambda) * (cos(pi * l / (L-1)) + 1) / 2 + lambda,  l = 0..L-1
 *   t_l  = ceil(r(l) * M), clamped to [1, M]  (L = 1 gives r = 1)
 * Returns t_l, or DYMOE_EINVAL for layer outside [0,L), lambda outside [0,1],
 * M < 1 or L < 1.
 */
int dymoe_depth_schedule(int layer, int n_layers, double lambda, int M);

/*
 * Bit-width per expert (paper Sec. 1, Sec. 4.3, Sec. 5: the top-t_l experts by
 * importance are critical and keep high precision, the rest get low precision
 * or 0 bits = skipped).  Generalised to an ordered tier table.
 * Experts are ranked by (importance descending, load descending, index
 * ascending); rank positions [0,c0) get tier_bits[0], the next c1 get
 * tier_bits[1], ...; then bits[e] = max(tier bits, floor_bits).
 * importance [E]: int32 for DYMOE_PHASE_PREFILL, fp32 for DYMOE_PHASE_DECODE.
 * load [E] int32 or NULL.  tier_count / tier_bits: HOST arrays of n_tiers
 * entries (1 <= n_tiers <= DYMOE_MAX_TIERS), counts >= 0 summing to E, bits in
 * {0,2,4,8,16}.  bits [E] uint8, rank [E] int32 (position of expert e) or NULL.
 * The two-tier paper mode is tier_count = {t_l, E - t_l}.
 */
int dymoe_assign_precision(dymoe_ctx* ctx, int phase, const void* importance,
                           const int32_t* load, int E, int n_tiers,
                           const int32_t* tier_count, const uint8_t* tier_bits, int floor_bits,
                           uint8_t* bits, int32_t* rank, void* stream);

/*
 * Decode-step front end: dymoe_route_topk, dymoe_expert_importance (decode
 * phase: importance = gate score, Sec. 4.2.2 Eq. 3) and dymoe_assign_precision
 * (Sec. 4.3, Sec. 5) in one launch, for steps of 1 <= T <= DYMOE_FRONT_MAX_TOKENS
 * tokens, where three dependent launches of microseconds each would cost more
 * than their work.  Arguments have the meaning, layout and limits they have in
 * the three calls (importance: [E] fp32; probs may be NULL; rank may be NULL;
 * tier_count / tier_bits: host arrays read before the launch), and every
 * output is bit for bit what the three calls in turn produce.  With a router
 * of 256 KiB or more (E * H * 2 bytes) and a probs buffer, the logits are
 * computed by a launch of their own over many workgroups and handed to the
 * finishing launch through probs (two launches; same outputs).
 */
int dymoe_decode_front(dymoe_ctx* ctx, const void* x, const void* wg, const float* bias,
                       int T, int H, int E, int k, int renorm, int n_tiers,
                       const int32_t* tier_count, const uint8_t* tier_bits, int floor_bits,
                       int32_t* idx, float* w, float* probs, float* importance, int32_t* load,
                       uint8_t* bits, int32_t* rank, void* stream);

/*
 * Group-wise asymmetric quantize-and-pack of one matrix (the paper, Sec. 5,
 * quantizes expert weights only and leaves the base quantizer exchangeable;
 * this is round-to-nearest with the group minimum as zero point).
 * For every row and every group of `group` consecutive columns, in binary32
 * with one correctly rounded operation per step:
 *   lo = min, hi = max over the group
 *   zero  = fp16(lo)                     m = (float)zero
 *   scale = fp16((hi - lo) / (2^bits-1)) s = (float)scale
 *   inv   = s > 0 ? 1/s : 0
 *   q     = clamp(rint((w - m) * inv), 0, 2^bits-1)
 * Codes are packed little-endian along the row: code j of a byte sits at bit
 * bits*j (int4: byte = q[2i] | q[2i+1]<<4; int2: four codes per byte; int8: one).
 * The dequantised weight is s*q + m.
 * w [N,K] bf16 (finite, magnitude within fp16 range), codes [N, K*bits/8],
 * scale and zero [N, K/group] fp16.  bits in {2,4,8}; group = 64; K multiple of
 * group; w and codes 16-byte aligned.
 */
int dymoe_quantize_pack(dymoe_ctx* ctx, const void* w, long N, long K, int bits, int group,
                        uint8_t* codes, void* scale, void* zero, void* stream);

/*
 * Error-compensated quantize-and-pack (the paper, Sec. 5, quantizes the experts
 * with GPTQ as its base algorithm; the published algorithm, restated).  Same
 * outputs and formats as dymoe_quantize_pack, row-major, so the FFN reads them
 * unchanged.  A row is quantised column by column; with U the upper triangular
 * factor of the inverse of the damped Hessian of the calibration inputs,
 * H^-1 = U^T U, in binary32, one correctly rounded operation per step, columns
 * c in ascending order, v the row widened to fp32:
 *   at the first column of a group: lo, hi, zero, scale, m, s, inv from the
 *     group's current values, as in dymoe_quantize_pack
 *   q  = clamp(rint((v[c] - m) * inv), 0, 2^bits-1)
 *   dq = (float)q * s;  dq = dq + m
 *   e  = (v[c] - dq) / U[c,c]
 *   v[j] = fma(-e, U[c,j], v[j])          for every j > c
 * u [K,K] fp32 row-major, device, 16-byte aligned (only the upper triangle is
 * read; U[c,c] > 0); from dymoe_gptq_factor or the caller's own.  The identity
 * gives dymoe_quantize_pack's result.  workspace: dymoe_gptq_workspace_bytes(N,
 * K) bytes of device memory, 256-byte aligned (an fp32 copy of the matrix and
 * 128 errors per row); its contents are garbage afterwards.  Other arguments,
 * limits and errors as dymoe_quantize_pack; DYMOE_ENOSPC if the workspace is
 * too small.  Enqueues about 2 K/64 launches on `stream`; never synchronises.
 */
/*
 * The two steps before it (GPTQ as published; Sec. 5 of the paper only names it).
 * dymoe_gptq_hessian: hess (+)= X^T X over calibration inputs x [n, K] bf16 (rows
 * = tokens entering the matrix), hess [K, K] fp32 row-major, both device, 16-byte
 * aligned; accumulate = 0 overwrites, 1 adds to what hess holds (several batches).
 * bf16 products are exact, sums are fp32 on the matrix cores.  K multiple of 8,
 * K <= 65536.
 * dymoe_gptq_factor: u = the upper triangular U with (H + lambda I)^-1 = U^T U,
 * lambda = damp * mean(diag H); a diagonal entry that is exactly zero (a column
 * no input ever reached) counts as 1 and becomes 1 (+ lambda).  fp32 throughout.
 * hess is read only; u [K, K] fp32, fully written (zeros below the diagonal);
 * workspace of dymoe_gptq_factor_workspace_bytes(K) bytes (two K x K fp32
 * matrices and change), 256-byte aligned.  K multiple of 64, K <= 65536, damp >=
 * 0 (the published default is 0.01).  H + lambda I must be positive definite in
 * fp32 (a square root of a negative pivot gives NaNs in u, nothing is checked).
 * Errors as elsewhere; both enqueue on `stream` and return without waiting.
 */
int dymoe_gptq_hessian(dymoe_ctx* ctx, const void* x, long n, long K, int accumulate, float* hess, void* stream);
size_t dymoe_gptq_factor_workspace_bytes(long K);
int dymoe_gptq_factor(dymoe_ctx* ctx, const float* hess, long K, float damp, float* u, void* workspace,
                      size_t workspace_bytes, void* stream);
size_t dymoe_gptq_workspace_bytes(long N, long K);
int dymoe_gptq_quantize_pack(dymoe_ctx* ctx, const void* w, const float* u, long N, long K, int bits, int group,
                             uint8_t* codes, void* scale, void* zero, void* workspace, size_t workspace_bytes,
                             void* stream);

/*
 * Device-driven quantization of a layer's experts, so that the precision
 * decision never travels to the host: for each expert e with bits[e] in {2,4,8}
 * (and load[e] > 0 when load is given), quantize table[e].w[0..3) at bits[e]
 * into table[e].q8/s8/z8, q4/s4/z4 or q2/s2/z2 (same arithmetic as dymoe_quantize_pack;
 * layout = DYMOE_LAYOUT_ROWMAJOR or DYMOE_LAYOUT_TILE, the latter needs H and F
 * multiples of 128).  Experts at 16 or 0 bits are left untouched.
 * table [E] device, bits [E] uint8 device, load [E] int32 device or NULL.
 * Weight and code pointers in the table must be 16-byte aligned.
 */
int dymoe_quantize_experts(dymoe_ctx* ctx, const dymoe_expert_fmt* table, const uint8_t* bits,
                           const int32_t* load, int E, int H, int F, int group, int layout,
                           void* stream);

/*
 * bf16 row-major [N,K] -> bf16 tile layout (see dymoe_expert_fmt), a pure
 * permutation done once when an expert's weights are loaded.  N multiple of
 * 32, K multiple of 128; w and tiles 16-byte aligned, distinct buffers.
 */
int dymoe_pack_tiles(dymoe_ctx* ctx, const void* w, long N, long K, void* tiles, void* stream);

/*
 * The same for a quantised matrix: codes [N, K*bits/8] with scale and zero
 * [N, K/64] as dymoe_quantize_pack and dymoe_gptq_quantize_pack write them ->
 * the tile layout the GEMM path reads (what dymoe_quantize_experts writes with
 * DYMOE_LAYOUT_TILE), so that an expert quantised off-line (Sec. 5) serves
 * prefill as well.  A pure permutation.  bits in {2,4,8}; N multiple of 32, K
 * multiple of 128; code buffers 16-byte aligned; source and destination distinct.
 */
int dymoe_pack_code_tiles(dymoe_ctx* ctx, const uint8_t* codes, const void* scale, const void* zero, long N, long K,
                          int bits, uint8_t* t_codes, void* t_scale, void* t_zero, void* stream);

/*
 * Mixed-precision SwiGLU expert FFN (paper Sec. 4.1: the executor runs the
 * layer on a unified mixed-precision weight set; Sec. 1: a 0-bit expert is
 * skipped):
 *   y[t,:] = sum_{slot<k} w[t,slot] * W2_e( silu(W1_e x_t) * (W3_e x_t) ),
 *   e = idx[t,slot], each expert's weights taken at bits[e]: 16 = table[e].w,
 *   8 / 4 / 2 = the dequantised q8 / q4 / q2 codes, 0 = term omitted (no renormalising).
 * x [T,H] bf16, idx [T,k] int32, w [T,k] fp32, bits [E] uint8, table [E].
 * y [T,H] bf16 (DYMOE_OUT_BF16) or fp32 (DYMOE_OUT_F32); every row is written.
 * path: DYMOE_PATH_AUTO picks GEMV for T <= 4 (or when the sizes rule out the
 * GEMM), GEMM otherwise.  GEMV reads the codes in DYMOE_LAYOUT_ROWMAJOR, GEMM in
 * DYMOE_LAYOUT_TILE.
 * workspace: at least dymoe_workspace_bytes(T,H,F,E,k) bytes, 256-byte aligned;
 * contents are scratch.  Limits: group = 64; H, F multiples of 64;
 * GEMV path H <= 8192; GEMM path H, F multiples of 128; E <= DYMOE_MAX_EXPERTS.
 * Activations and the SwiGLU intermediate must stay inside fp16 range.
 * Every sum is taken in a fixed order (no atomics): the same inputs give the
 * same bits from launch to launch, on either path.
 */
int dymoe_moe_ffn_mixed(dymoe_ctx* ctx, const void* x, const int32_t* idx, const float* w,
                        const uint8_t* bits, const dymoe_expert_fmt* table,
                        int T, int H, int F, int E, int k, int group, int out_dtype, int path,
                        void* y, void* workspace, size_t workspace_bytes, void* stream);

/*
 * A whole decode step on resident formats in two launches: dymoe_decode_front
 * (Sec. 4.2.2 Eq. 3 importance, Sec. 4.3 assignment) and dymoe_moe_ffn_mixed on its
 * GEMV path (Sec. 4.1: the executor on the mixed-precision weight set), with the
 * front end worked out by every workgroup of the FFN's first launch for itself
 * instead of by a launch of its own: a decode layer is a few tens of microseconds
 * of weight streaming, and a launch boundary plus the front end's own chain of
 * memory latencies is a tenth of that.  Arguments, layouts, limits and errors are
 * those of the two calls; every output (idx, w, probs, importance, load, bits,
 * rank, y) holds bit for bit what dymoe_decode_front followed by
 * dymoe_moe_ffn_mixed(path = DYMOE_PATH_GEMV) writes.  The formats the assignment
 * may name must already be materialised in `table` (row-major codes).
 * DYMOE_ENOTSUP outside T <= 4, E <= 64, k <= 8, H a multiple of 64 up to 8192:
 * the caller then makes the two calls.
 */
int dymoe_decode_step(dymoe_ctx* ctx, const void* x, const void* wg, const float* bias, int T, int H, int F,
                      int E, int k, int renorm, int n_tiers, const int32_t* tier_count, const uint8_t* tier_bits,
                      int floor_bits, const dymoe_expert_fmt* table, int group, int out_dtype, int32_t* idx,
                      float* w, float* probs, float* importance, int32_t* load, uint8_t* bits, int32_t* rank,
                      void* y, void* workspace, size_t workspace_bytes, void* stream);

/*
 * Diagnostic (tests, profiling): where the grouped-GEMM path of dymoe_moe_ffn_mixed leaves its token
 * grouping in the workspace, so that a caller can see which (token, slot) pair went to which row of which
 * tile (paper Sec. 4.2.1: the per-expert token lists Tokens_j).  Returns the byte offset of an int32 array
 * laid out as counts[E] | offsets[E+1] | (E ints: the first E bytes hold the bit width each expert is run at) | ntiles, pairs, experts with tiles (+5 unused) | perm[T*k]:
 * counts[e] = pairs routed to expert e at a non-zero precision, offsets = their exclusive prefix sums,
 * perm[offsets[e] + i] = the i-th pair (token * k + slot) of expert e, in the order the GEMM's tiles take
 * them (rows [128 j, 128 j + 128) of an expert form its j-th tile).  Pure host function; 0 for invalid sizes.
 */
size_t dymoe_ffn_plan_offset(int T, int H, int F, int E, int k);

/*
 * dymoe_moe_ffn_mixed for callers that cannot allocate device memory or hand in
 * a workspace (code under HIP graph capture, tight serving loops, harnesses that
 * forbid hipMalloc).  Same arguments, results, limits and errors, minus the
 * workspace: its scratch is a fixed array of DYMOE_STATIC_SCRATCH_BYTES that the
 * library keeps in each GPU's memory from the moment it is loaded until the
 * process ends.  The call allocates and frees nothing, on the device or through
 * any allocating runtime routine, and records no timing events (per-kernel
 * timing is off for its launches).
 *  - DYMOE_ENOSPC when dymoe_workspace_bytes(T,H,F,E,k) exceeds
 *    DYMOE_STATIC_SCRATCH_BYTES (8 MiB: a Mixtral-shaped decode step of up to 16
 *    tokens takes 5.5 MiB; prefill batches need the workspace form).
 *  - Every call on a GPU shares that GPU's array: calls that overlap in time on
 *    one GPU (different streams, different threads) race; calls on one stream do
 *    not.  Nothing in it has to start at zero (each launch writes what it later
 *    reads), so the previous call's contents are harmless.
 *  - The array's address is taken once per device in dymoe_create; the context
 *    must have been created for the device the call runs on.
 */
#define DYMOE_STATIC_SCRATCH_BYTES (8u << 20)
int dymoe_moe_ffn_mixed_noalloc(dymoe_ctx* ctx, const void* x, const int32_t* idx, const float* w,
                                const uint8_t* bits, const dymoe_expert_fmt* table,
                                int T, int H, int F, int E, int k, int group, int out_dtype, int path,
                                void* y, void* stream);

/*
 * Host-resident experts (Sec. 4.4.1, Phase-Adaptive Prefetcher): the weights a
 * later layer is predicted to need are copied from pinned host memory into
 * device buffers on a side stream while the compute stream works on the current
 * layer.  Which experts to fetch is decided with the calls above: Eq. 6 applies
 * the NEXT layer's router to the current hidden state (dymoe_route_topk with
 * that layer's wg); decode prefetches its top-t experts (Eq. 8: call it with
 * k = t); prefill counts the predicted activations per expert (Eq. 7: the load
 * histogram of dymoe_expert_importance) and takes the t most frequent
 * (dymoe_assign_precision with tiers (t, E - t) marks them).
 *
 * dymoe_prefetch_submit: enqueue on side_stream the copy of `bytes` from
 * host_pinned_src (pinned host memory, owned by the caller, must stay valid and
 * unchanged until the copy has completed) to dev_dst (device), followed by an
 * event; *event_out receives the event (opaque, owned by the caller until
 * dymoe_prefetch_release).  bytes == 0 records only the event.  Does not block.
 * dymoe_prefetch_wait: work enqueued on compute_stream after this call starts
 * only when the copy behind `event` has completed.  Does not block the host.
 * dymoe_prefetch_done: 1 if the copy has completed, 0 if not yet (host query).
 * dymoe_prefetch_release: destroy the event (its copy may still be running).
 * Errors: DYMOE_EINVAL, DYMOE_ENOCTX, DYMOE_EHIP.
 */
int dymoe_prefetch_submit(dymoe_ctx* ctx, const void* host_pinned_src, void* dev_dst, size_t bytes,
                          void* side_stream, void** event_out);
int dymoe_prefetch_wait(dymoe_ctx* ctx, void* event, void* compute_stream);
int dymoe_prefetch_done(dymoe_ctx* ctx, void* event);
int dymoe_prefetch_release(dymoe_ctx* ctx, void* event);

/*
 * Glue between the layers of an expert-only stack (not from the paper, which
 * runs whole transformer blocks): v = h[t,:] + alpha * y[t,:], h_out[t,:] =
 * bf16(v / rms(v)), fp32 arithmetic (fma, then sum of squares by lane and a
 * cross-lane sum).  h, h_out: [T,H] bf16 (may alias); y: [T,H] bf16 or fp32
 * (y_dtype = DYMOE_OUT_BF16 / DYMOE_OUT_F32).  A row of zeros stays zero.
 */
int dymoe_residual_rmsnorm(dymoe_ctx* ctx, const void* h, const void* y, int y_dtype, float alpha,
                           int T, int H, void* h_out, void* stream);

/*
 * Measurement aid, not a step of the method: copies `bytes` (a multiple of
 * 16; src and dst 16-byte aligned device pointers that do not overlap) with
 * the access pattern of the weight-streaming kernels (16 bytes per lane,
 * 1 KiB per wavefront instruction).  Its traffic is exactly `bytes` read and
 * `bytes` written, which gives a profiler's HBM byte counters a known
 * quantity to be scaled by, and the rate it reaches is the copy rate the
 * machine sustains, the practical ceiling beside the 8 TB/s on the data sheet
 * (the paper's own evaluation reports latency only, Sec. 6.1 "Key Metrics").
 */
int dymoe_stream_copy(dymoe_ctx* ctx, const void* src, void* dst, size_t bytes, void* stream);

/*
 * Measurement aid, not a step of the method: a register-only loop of
 * v_mfma_f32_32x32x16_bf16, `iters` rounds of four independent accumulators in
 * every wavefront, one (waves_per_simd = 1) or two wavefronts on every SIMD of
 * the chip, no memory traffic but one float per thread at the end (sink: device,
 * at least 512 * compute units floats; sink_floats its length).  *flops (host
 * pointer, may be NULL) receives the floating-point operations of the launch;
 * time it with dymoe_timing_enable (kernel id 20).  The rate it sustains is the
 * matrix rate the chip reaches at the clock it holds under that load: the
 * practical ceiling of the prefill GEMM beside the data sheet's 2.5 PFLOP/s
 * (the paper gives no kernel-level figure, Sec. 6.1 "Key Metrics").
 */
int dymoe_mfma_peak(dymoe_ctx* ctx, int iters, int waves_per_simd, float* sink, size_t sink_floats, double* flops,
                    void* stream);

/*
 * Mixed-precision expert cache with one byte budget (paper Sec. 4.4.2): host-side
 * bookkeeping for a caller that keeps experts in an arena of device memory.  No
 * GPU call is made and no device memory is touched; all pointers are host pointers.
 * Rules: No Duplication (an expert is resident in one format at most), Precision
 * Promotion (a request above the resident precision loads the higher format and
 * drops the lower one), Conservative Reuse (a request at or below the resident
 * precision is a hit and the resident format is used).
 * dymoe_cache_create: formats format_bits[i] in {2,4,8,16} (distinct), each with
 *   the bytes one expert takes in it.  The arena is cut into blocks of the
 *   largest slot size (rounded up to 256 bytes); a block serves one format at a
 *   time and holds as many of its slots as fit.  DYMOE_ENOSPC: the budget holds
 *   no block; DYMOE_ENOTSUP: more than DYMOE_CACHE_MAX_EVICT slots per block.
 * dymoe_cache_request: the expert `key` is wanted at `want_bits`.  On return
 *   out->offset is the byte offset of its slot in the arena, out->use_bits the
 *   precision to run it at, out->load_bits the format the caller has to copy
 *   into the slot (0: nothing), out->evicted[0..n_evicted) the keys that lost
 *   their slots, out->dropped_offset the slot a promotion freed (else -1).
 *   Room is taken from a free slot, a free block, or else the least recently
 *   used of (a) the residents of the requested format and (b) whole blocks of
 *   other formats (a block is as recent as its most recent resident); keys in
 *   protect[0..n_protect) are never evicted.  DYMOE_ENOSPC: nothing evictable;
 *   the cache is then unchanged.
 * dymoe_cache_lookup: 1 and the resident format / offset, or 0.
 * dymoe_cache_set_cyclic, dymoe_cache_request_at: an eviction order for callers whose requests walk a cyclic
 *   schedule of n_positions positions (the layers of a decoder stack, visited 0 .. L-1 in every step).  The paper
 *   extends the standard LRU cache; when one pass of the schedule asks for more experts than the cache holds, LRU
 *   order evicts every entry shortly before its position comes round again.  With n_positions > 0 the request says
 *   at which position it is made (0 <= position < n_positions), every resident remembers the position it was last
 *   asked for at, and "least recently used" is replaced by "its position comes up last, counted from the request's"
 *   (a resident of the request's own position that is not being asked for is a whole cycle away; least recently
 *   used among equals), for residents and for blocks alike (a block ranks with the resident of its that would go
 *   last).  The three rules, protection and the unchanged-on-failure guarantee are the same.  n_positions = 0
 *   (the default) restores LRU order; dymoe_cache_request is dymoe_cache_request_at at the position of the request
 *   before it.  DYMOE_EINVAL: negative n_positions, position out of range.
 * dymoe_cache_create_pools: the same rules over a fixed partition instead of one budget: slot_counts[i] >= 1 slots
 *   of format_bits[i], laid out format after format (offsets are into an arena of dymoe_cache_block_bytes bytes,
 *   slot j of format i after all slots of the formats before it); a slot never serves another format, so room for a
 *   request comes from free or least recently used unprotected slots of its own format only.
 */
typedef struct dymoe_cache dymoe_cache;
#define DYMOE_CACHE_MAX_FORMATS 4
#define DYMOE_CACHE_MAX_EVICT 16
#define DYMOE_CACHE_HIT 0
#define DYMOE_CACHE_MISS 1
#define DYMOE_CACHE_PROMOTE 2
typedef struct {
    int32_t kind;
    int32_t use_bits;
    int32_t load_bits;
    int32_t n_evicted;
    int64_t offset;
    int64_t dropped_offset;
    int64_t evicted[DYMOE_CACHE_MAX_EVICT];
} dymoe_cache_action;
int dymoe_cache_create(dymoe_cache** out, size_t budget_bytes, int n_formats, const int32_t* format_bits,
                       const size_t* slot_bytes);
int dymoe_cache_create_pools(dymoe_cache** out, int n_formats, const int32_t* format_bits, const size_t* slot_bytes,
                             const int32_t* slot_counts);
void dymoe_cache_destroy(dymoe_cache* cache);
int dymoe_cache_request(dymoe_cache* cache, int64_t key, int want_bits, const int64_t* protect, int n_protect,
                        dymoe_cache_action* out);
int dymoe_cache_set_cyclic(dymoe_cache* cache, int n_positions);
int dymoe_cache_request_at(dymoe_cache* cache, int64_t key, int want_bits, const int64_t* protect, int n_protect,
                           int position, dymoe_cache_action* out);
int dymoe_cache_lookup(const dymoe_cache* cache, int64_t key, int32_t* bits, int64_t* offset);
size_t dymoe_cache_block_bytes(const dymoe_cache* cache);
size_t dymoe_cache_bytes_resident(const dymoe_cache* cache);

/*
 * Per-kernel timing (diagnostic; the paper reports only end-to-end latency,
 * Sec. 6.1 "Key Metrics", so these serve the roofline accounting).
 * dymoe_timing_enable: launches of the kernels whose bit is set in kernel_mask
 * (bit i = kernel id i, ids 0..21 in the order route, token_norm, importance,
 * assign, quantize, gemv_phase1, gemv_phase2, gemv_combine, plan, gemm1, gemm2,
 * gemm_combine, stream_copy, decode_front, attn_stats, attn_colsum, gptq_group,
 * gptq_trail, gptq_hessian, gptq_factor, mfma_peak, route_select; gemv_combine is reserved: the decode path's
 * second phase writes y itself and no launch carries that id; route_select is the second of the two launches
 * dymoe_route_topk makes when it cuts the logits by experts as well as by tokens, route then names the first) carry a start and a stop HIP event on the dispatch itself, so
 * the interval is the kernel's execution time on the launch stream; 0 switches
 * timing off.  Either way, records not yet read are dropped.
 * dymoe_timing_read: waits for the recorded launches of `kernel`, drops their records and returns
 * their summed duration in milliseconds and their count (host pointers).
 * Do not enable timing while the stream is being captured into a graph.
 * dymoe_kernel_name: the kernel's name as a profiler shows it, NULL if unknown.
 */
int dymoe_timing_enable(dymoe_ctx* ctx, unsigned kernel_mask);
int dymoe_timing_read(dymoe_ctx* ctx, int kernel, double* total_ms, int* launches);
const char* dymoe_kernel_name(int kernel);

#ifdef __cplusplus
}
#endif
#endif /* DYMOE_H */
