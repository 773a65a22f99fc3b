/*
 * DyMoE mixed-precision MoE layer: CPU oracle.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, single-threaded, plain
 * reference that the GPU library is checked against.  It shares no code,
 * header, table or helper with the HIP path and must never be linked,
 * imported or called from the product path (only tests, the smoke check and
 * the CPU-baseline leg of the benchmark use it).
 *
 * Arithmetic: fp64 for every step that is real arithmetic (routing, softmax,
 * importance scores, schedule, FFN).  The quantizer is the one step whose
 * output is an integer code decided by floating point, so it is written as an
 * exact sequence of IEEE-754 binary32 operations (no fusion) that the GPU must
 * reproduce bit for bit.
 *
 * Build: gcc -O2 -std=c11 -ffp-contract=off -fno-fast-math -fPIC -shared.
 *
 * Passages followed (DyMoE paper):
 *   routing              Sec. 2.1 (router picks a few experts per token) and
 *                        the gate form of Sec. 4.4.1 Eq. "g = Softmax(h W_g)",
 *                        "s = TopK_k(g)".
 *   prefill importance   Sec. 4.2.1, expert importance = number of
 *                        heavy-hitter tokens (top tokens by score s_i) that
 *                        are routed to the expert.
 *   decode importance    Sec. 4.2.2, importance = gating score g_j.
 *   retention schedule   Sec. 4.3, cosine schedule r(l) and t_l = ceil(r(l) M).
 *   tiering              Sec. 1 / Sec. 5: top-t_l experts critical (high
 *                        precision), the rest low precision or 0-bit (skipped).
 *   prefetch frequency   Sec. 4.4.1 token-frequency count c_e (same histogram
 *                        as the total load returned by the importance step).
 *   error-compensated   Sec. 5 (GPTQ as the base quantizer): see
 *   quantizer            oracle_gptq_quantize_pack.
 * The paper leaves the quantizer (it uses an off-line one and says the base
 * algorithm is exchangeable) and the expert FFN form unstated; this build
 * uses asymmetric group-wise round-to-nearest with fp16 scale and fp16 zero
 * (= group minimum) and a SwiGLU expert  W2( silu(W1 x) * (W3 x) ).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

/* ------------------------------------------------------------------ */
/* number formats                                                      */
/* ------------------------------------------------------------------ */

static float bf16_to_f32(uint16_t b)
{
    uint32_t u = (uint32_t)b << 16;
    float f;
    memcpy(&f, &u, 4);
    return f;
}

static float f16_to_f32(uint16_t h)
{
    uint32_t sign = (uint32_t)(h & 0x8000u) << 16;
    uint32_t exp = (h >> 10) & 0x1fu;
    uint32_t man = h & 0x3ffu;
    uint32_t u;
    if (exp == 0) {
        if (man == 0) {
            u = sign;
        } else { /* subnormal: man * 2^-24 */
            float f = (float)man * 5.9604644775390625e-8f; /* exact */
            memcpy(&u, &f, 4);
            u |= sign;
        }
    } else if (exp == 31) {
        u = sign | 0x7f800000u | (man << 13);
    } else {
        u = sign | ((exp + 112u) << 23) | (man << 13);
    }
    float f;
    memcpy(&f, &u, 4);
    return f;
}

/* binary32 -> binary16, round to nearest even, subnormals honoured */
static uint16_t f32_to_f16_rne(float f)
{
    uint32_t u;
    memcpy(&u, &f, 4);
    uint32_t sign = (u >> 16) & 0x8000u;
    uint32_t a = u & 0x7fffffffu;
    if (a >= 0x7f800000u) /* inf / nan */
        return (uint16_t)(sign | 0x7c00u | (a > 0x7f800000u ? 0x200u : 0u));
    int e = (int)(a >> 23) - 127;
    uint32_t man = a & 0x7fffffu;
    if (e > 15)
        return (uint16_t)(sign | 0x7c00u);
    if (e >= -14) {
        uint32_t h = ((uint32_t)(e + 15) << 10) | (man >> 13);
        uint32_t rem = man & 0x1fffu;
        if (rem > 0x1000u || (rem == 0x1000u && (h & 1u)))
            h++; /* carry may run into the exponent, up to inf */
        return (uint16_t)(sign | h);
    }
    if ((a >> 23) == 0)
        return (uint16_t)sign; /* binary32 subnormal: far below half of 2^-24 */
    /* result is a binary16 subnormal: units of 2^-24 */
    uint32_t full = man | 0x800000u; /* value = full * 2^(e-23) */
    int ts = 13 + (-14 - e);         /* shift that leaves units of 2^-24 */
    if (ts > 24)
        return (uint16_t)sign;
    uint32_t q = full >> ts;
    uint32_t rem = full & ((1u << ts) - 1u);
    uint32_t halfway = 1u << (ts - 1);
    if (rem > halfway || (rem == halfway && (q & 1u)))
        q++;
    return (uint16_t)(sign | q);
}

/* exported so that the tests can pin the conversions against numpy's */
uint16_t oracle_f32_to_f16(float f) { return f32_to_f16_rne(f); }
float oracle_f16_to_f32(uint16_t h) { return f16_to_f32(h); }
float oracle_bf16_to_f32(uint16_t b) { return bf16_to_f32(b); }

/* ------------------------------------------------------------------ */
/* sorting helper: full sort of indices by (key descending, index ascending) */
/* ------------------------------------------------------------------ */

typedef struct {
    double key;
    double key2;
    int index;
} sort_item;

static int cmp_desc(const void* pa, const void* pb)
{
    const sort_item* a = (const sort_item*)pa;
    const sort_item* b = (const sort_item*)pb;
    if (a->key > b->key) return -1;
    if (a->key < b->key) return 1;
    if (a->key2 > b->key2) return -1;
    if (a->key2 < b->key2) return 1;
    return (a->index > b->index) - (a->index < b->index);
}

/* ------------------------------------------------------------------ */
/* S1 routing: logits, softmax over all experts, top-k by full sort     */
/* ------------------------------------------------------------------ */

/*
 * x [T,H] bf16 bits, wg [E,H] bf16 bits, bias [E] or NULL.
 * logits [T,E], probs [T,E] (fp64, softmax over all E experts),
 * idx [T,k] (descending score, ties to the lower index), w [T,k]
 * (the selected probabilities, divided by their sum when renorm != 0).
 */
int oracle_route_topk(const uint16_t* x, const uint16_t* wg, const float* bias,
                      int T, int H, int E, int k, int renorm,
                      int32_t* idx, double* w, double* probs, double* logits)
{
    if (T < 0 || H <= 0 || E <= 0 || k <= 0 || k > E) return -1;
    sort_item* items = (sort_item*)malloc(sizeof(sort_item) * (size_t)E);
    double* lg = (double*)malloc(sizeof(double) * (size_t)E);
    double* pr = (double*)malloc(sizeof(double) * (size_t)E);
    for (int t = 0; t < T; t++) {
        for (int e = 0; e < E; e++) {
            double s = 0.0;
            for (int h = 0; h < H; h++)
                s += (double)bf16_to_f32(x[(size_t)t * H + h]) *
                     (double)bf16_to_f32(wg[(size_t)e * H + h]);
            if (bias) s += (double)bias[e];
            lg[e] = s;
        }
        double mx = lg[0];
        for (int e = 1; e < E; e++)
            if (lg[e] > mx) mx = lg[e];
        double den = 0.0;
        for (int e = 0; e < E; e++) {
            pr[e] = exp(lg[e] - mx);
            den += pr[e];
        }
        for (int e = 0; e < E; e++) pr[e] /= den;
        for (int e = 0; e < E; e++) {
            items[e].key = lg[e];
            items[e].key2 = 0.0;
            items[e].index = e;
        }
        qsort(items, (size_t)E, sizeof(sort_item), cmp_desc);
        double sel = 0.0;
        for (int j = 0; j < k; j++) sel += pr[items[j].index];
        for (int j = 0; j < k; j++) {
            idx[(size_t)t * k + j] = items[j].index;
            w[(size_t)t * k + j] = renorm ? pr[items[j].index] / sel : pr[items[j].index];
        }
        if (probs) memcpy(probs + (size_t)t * E, pr, sizeof(double) * (size_t)E);
        if (logits) memcpy(logits + (size_t)t * E, lg, sizeof(double) * (size_t)E);
    }
    free(items);
    free(lg);
    free(pr);
    return 0;
}

/* ------------------------------------------------------------------ */
/* S2 importance                                                       */
/* ------------------------------------------------------------------ */

/* activation-norm stand-in for the attention-derived token score:
 * s_t = sqrt(sum_h x[t,h]^2), fp64 */
void oracle_token_score_norm(const uint16_t* x, int T, int H, double* score)
{
    for (int t = 0; t < T; t++) {
        double s = 0.0;
        for (int h = 0; h < H; h++) {
            double v = (double)bf16_to_f32(x[(size_t)t * H + h]);
            s += v * v;
        }
        score[t] = sqrt(s);
    }
}

/*
 * Prefill (Sec. 4.2.1): T_imp = the k_hh tokens with the largest score
 * (ties to the lower token index); importance[e] = number of (token, slot)
 * pairs with token in T_imp routed to e; load[e] = the same count over all
 * tokens (also the token-frequency count of Sec. 4.4.1).
 * heavy [T] (optional) receives 1 for tokens in T_imp.
 */
int oracle_expert_importance_prefill(const int32_t* idx, const double* score,
                                     int T, int E, int k, int k_hh,
                                     int32_t* importance, int32_t* load, uint8_t* heavy)
{
    if (k_hh < 0 || k_hh > T) return -1;
    sort_item* items = (sort_item*)malloc(sizeof(sort_item) * (size_t)(T > 0 ? T : 1));
    uint8_t* in_imp = (uint8_t*)calloc((size_t)(T > 0 ? T : 1), 1);
    for (int t = 0; t < T; t++) {
        items[t].key = score[t];
        items[t].key2 = 0.0;
        items[t].index = t;
    }
    qsort(items, (size_t)T, sizeof(sort_item), cmp_desc);
    for (int j = 0; j < k_hh; j++) in_imp[items[j].index] = 1;
    for (int e = 0; e < E; e++) {
        importance[e] = 0;
        load[e] = 0;
    }
    for (int t = 0; t < T; t++)
        for (int s = 0; s < k; s++) {
            int e = idx[(size_t)t * k + s];
            if (e < 0 || e >= E) { free(items); free(in_imp); return -2; }
            load[e]++;
            if (in_imp[t]) importance[e]++;
        }
    if (heavy) memcpy(heavy, in_imp, (size_t)T);
    free(items);
    free(in_imp);
    return 0;
}

/* Decode (Sec. 4.2.2): importance[e] = gating score of expert e; with more
 * than one token in the step, the mean over the tokens (extension). */
void oracle_expert_importance_decode(const double* probs, int T, int E, double* importance)
{
    for (int e = 0; e < E; e++) {
        double s = 0.0;
        for (int t = 0; t < T; t++) s += probs[(size_t)t * E + e];
        importance[e] = (T > 0) ? s / (double)T : 0.0;
    }
}

/* ------------------------------------------------------------------ */
/* S3 depth schedule and tier assignment                               */
/* ------------------------------------------------------------------ */

/* Sec. 4.3: r(l) = (1-lambda) (cos(pi l/(L-1)) + 1)/2 + lambda, l = 0..L-1 */
double oracle_retention_ratio(int layer, int n_layers, double lambda)
{
    if (n_layers <= 1) return 1.0;
    const double pi = 3.14159265358979323846;
    return (1.0 - lambda) * (cos(pi * (double)layer / (double)(n_layers - 1)) + 1.0) / 2.0 + lambda;
}

/* Sec. 4.3: t_l = ceil(r(l) * M); the product is nudged down by 1e-9 so that
 * a mathematically integral product that lands one ulp above the integer is
 * not rounded up; clamped to [1, M]. */
int oracle_depth_schedule(int layer, int n_layers, double lambda, int M)
{
    if (M <= 0 || n_layers <= 0 || layer < 0 || layer >= n_layers || lambda < 0.0 || lambda > 1.0)
        return -1;
    double v = oracle_retention_ratio(layer, n_layers, lambda) * (double)M;
    int t = (int)ceil(v - 1e-9);
    if (t < 1) t = 1;
    if (t > M) t = M;
    return t;
}

/*
 * Rank experts by (importance desc, load desc, index asc) with a full sort;
 * rank position -> tier through the cumulative tier counts; bits = max(tier
 * bits, floor_bits).  rank[e] = position of expert e in the order.
 */
int oracle_assign_precision(const double* importance, const int32_t* load, int E,
                            int n_tiers, const int32_t* tier_count, const uint8_t* tier_bits,
                            int floor_bits, uint8_t* bits, int32_t* rank)
{
    long total = 0;
    for (int i = 0; i < n_tiers; i++) {
        if (tier_count[i] < 0) return -1;
        total += tier_count[i];
    }
    if (total != E) return -1;
    sort_item* items = (sort_item*)malloc(sizeof(sort_item) * (size_t)E);
    for (int e = 0; e < E; e++) {
        items[e].key = importance[e];
        items[e].key2 = load ? (double)load[e] : 0.0;
        items[e].index = e;
    }
    qsort(items, (size_t)E, sizeof(sort_item), cmp_desc);
    int tier = 0, left = n_tiers > 0 ? tier_count[0] : 0;
    for (int pos = 0; pos < E; pos++) {
        while (left == 0) {
            tier++;
            left = tier_count[tier];
        }
        left--;
        int e = items[pos].index;
        int b = tier_bits[tier];
        if (b < floor_bits) b = floor_bits;
        bits[e] = (uint8_t)b;
        rank[e] = pos;
    }
    free(items);
    return 0;
}

/* ------------------------------------------------------------------ */
/* S4 group-wise asymmetric quantize-and-pack                          */
/* ------------------------------------------------------------------ */

/*
 * w [N,K] bf16 bits.  For each row and each group of `group` consecutive
 * columns, in binary32 (each line one correctly rounded operation):
 *   lo = min, hi = max
 *   zero  = fp16(lo)                 m = (float)zero
 *   scale = fp16((hi - lo) / qmax)   s = (float)scale
 *   inv   = s > 0 ? 1 / s : 0
 *   q     = clamp((int)rint((w - m) * inv), 0, qmax)
 * codes packed little-endian along the row: code j of a byte sits at bit
 * position bits*j.  codes [N, K*bits/8], scale/zero [N, K/group] fp16 bits.
 */
int oracle_quantize_pack(const uint16_t* w, long N, long K, int bits, int group,
                         uint8_t* codes, uint16_t* scale, uint16_t* zero)
{
    if ((bits != 2 && bits != 4 && bits != 8) || group <= 0 || K % group != 0) return -1;
    const int per_byte = 8 / bits;
    if (group % per_byte != 0) return -1;
    const int qmax = (1 << bits) - 1;
    const long G = K / group;
    memset(codes, 0, (size_t)(N * K * bits / 8));
    for (long n = 0; n < N; n++) {
        for (long g = 0; g < G; g++) {
            const uint16_t* src = w + n * K + g * group;
            float lo = bf16_to_f32(src[0]);
            float hi = lo;
            for (int i = 1; i < group; i++) {
                float v = bf16_to_f32(src[i]);
                if (v < lo) lo = v;
                if (v > hi) hi = v;
            }
            uint16_t zh = f32_to_f16_rne(lo);
            float range = hi - lo;
            float step = range / (float)qmax;
            uint16_t sh = f32_to_f16_rne(step);
            float m = f16_to_f32(zh);
            float s = f16_to_f32(sh);
            float inv = (s > 0.0f) ? (1.0f / s) : 0.0f;
            scale[n * G + g] = sh;
            zero[n * G + g] = zh;
            for (int i = 0; i < group; i++) {
                float d = bf16_to_f32(src[i]) - m;
                float r = rintf(d * inv);
                int q = (int)r;
                if (q < 0) q = 0;
                if (q > qmax) q = qmax;
                long col = g * group + i;
                codes[n * (K * bits / 8) + col / per_byte] |=
                    (uint8_t)(q << (bits * (int)(col % per_byte)));
            }
        }
    }
    return 0;
}

/*
 * Error-compensated variant of the quantizer (paper Sec. 5: the experts are
 * quantised with GPTQ, "the basic quantization algorithm" of the paper's
 * implementation; the published algorithm is followed, restated here).
 *
 * A row of W is quantised column by column.  What rounding takes away from
 * column c is spread over the columns not yet quantised so that the layer
 * output on the calibration inputs changes least: with H = X^T X (+ damping)
 * the Hessian of that error and U the upper triangular factor of its inverse,
 * H^-1 = U^T U, the correction of column j > c is  -e U[c,j],  e = (w_c -
 * dequant(q_c)) / U[c,c].  Scale and zero of a group are fixed when its first
 * column is reached, from the row's current (already corrected) values, by
 * the same rule as the plain quantizer above; so are the codes.
 *
 * Like the plain quantizer this is an exact sequence of binary32 operations
 * (each line one correctly rounded operation, the correction one fused
 * multiply-add per column pair, columns c in ascending order):
 *   v[0..K) = (float) w[n, :]
 *   for each group g, columns base .. base + group - 1:
 *     lo, hi = min, max of v over the group;   zero, scale, m, s, inv as above
 *     for c in the group:
 *       q  = clamp(rint((v[c] - m) * inv), 0, qmax)
 *       dq = (float)q * s;  dq = dq + m
 *       e  = (v[c] - dq) / U[c,c]
 *       v[j] = fma(-e, U[c,j], v[j])   for j = c+1 .. K-1
 * u [K,K] fp32 row-major (only the upper triangle is read).  Outputs as
 * oracle_quantize_pack.
 */
int oracle_gptq_quantize_pack(const uint16_t* w, long N, long K, int bits, int group, const float* u,
                              uint8_t* codes, uint16_t* scale, uint16_t* zero)
{
    if ((bits != 2 && bits != 4 && bits != 8) || group <= 0 || K % group != 0) return -1;
    const int per_byte = 8 / bits;
    if (group % per_byte != 0) return -1;
    const int qmax = (1 << bits) - 1;
    const long G = K / group;
    float* v = (float*)malloc((size_t)K * sizeof(float));
    if (!v) return -2;
    memset(codes, 0, (size_t)(N * K * bits / 8));
    for (long n = 0; n < N; n++) {
        for (long j = 0; j < K; j++) v[j] = bf16_to_f32(w[n * K + j]);
        for (long g = 0; g < G; g++) {
            const long base = g * group;
            float lo = v[base];
            float hi = lo;
            for (int i = 1; i < group; i++) {
                if (v[base + i] < lo) lo = v[base + i];
                if (v[base + i] > hi) hi = v[base + i];
            }
            uint16_t zh = f32_to_f16_rne(lo);
            float range = hi - lo;
            float step = range / (float)qmax;
            uint16_t sh = f32_to_f16_rne(step);
            float m = f16_to_f32(zh);
            float s = f16_to_f32(sh);
            float inv = (s > 0.0f) ? (1.0f / s) : 0.0f;
            scale[n * G + g] = sh;
            zero[n * G + g] = zh;
            for (int i = 0; i < group; i++) {
                const long c = base + i;
                float d = v[c] - m;
                float r = rintf(d * inv);
                if (r < 0.0f) r = 0.0f;
                if (r > (float)qmax) r = (float)qmax;
                int q = (int)r;
                codes[n * (K * bits / 8) + c / per_byte] |= (uint8_t)(q << (bits * (int)(c % per_byte)));
                float dq = r * s;
                dq = dq + m;
                float e = (v[c] - dq) / u[c * K + c];
                for (long j = c + 1; j < K; j++) v[j] = fmaf(-e, u[c * K + j], v[j]);
            }
        }
    }
    free(v);
    return 0;
}

/* dequantised value of one element: s*q + m in fp64 (exact) */
static double dequant_at(const uint8_t* codes, const uint16_t* scale, const uint16_t* zero,
                         long K, int bits, int group, long n, long col)
{
    const int per_byte = 8 / bits;
    const int qmax = (1 << bits) - 1;
    uint8_t byte = codes[n * (K * bits / 8) + col / per_byte];
    int q = (byte >> (bits * (int)(col % per_byte))) & qmax;
    long G = K / group;
    double s = (double)f16_to_f32(scale[n * G + col / group]);
    double m = (double)f16_to_f32(zero[n * G + col / group]);
    return s * (double)q + m;
}

void oracle_dequantize(const uint8_t* codes, const uint16_t* scale, const uint16_t* zero,
                       long N, long K, int bits, int group, double* out)
{
    for (long n = 0; n < N; n++)
        for (long c = 0; c < K; c++)
            out[n * K + c] = dequant_at(codes, scale, zero, K, bits, group, n, c);
}

/* ------------------------------------------------------------------ */
/* S5 mixed-precision SwiGLU expert FFN                                */
/* ------------------------------------------------------------------ */

/* one row of an expert matrix at the expert's precision, widened to fp64 */
static void fetch_row(int bits, const uint16_t* wb, const uint8_t* codes,
                      const uint16_t* scale, const uint16_t* zero,
                      long K, int group, long n, double* row)
{
    if (bits == 16) {
        for (long c = 0; c < K; c++) row[c] = (double)bf16_to_f32(wb[n * K + c]);
    } else {
        for (long c = 0; c < K; c++) row[c] = dequant_at(codes, scale, zero, K, bits, group, n, c);
    }
}

/*
 * y[t,:] = sum_slot w[t,slot] * W2_e( silu(W1_e x_t) * (W3_e x_t) ),
 * e = idx[t,slot], each expert at precision bits[e]: 16 = the bf16 weights,
 * 8/4/2 = dequantised codes, 0 = term omitted (expert skipped).
 * Pointer tables have 3 entries per expert in the order W1 [F,H], W3 [F,H],
 * W2 [H,F]; an entry may be NULL when the expert's precision does not use it.
 * No intermediate is rounded; everything is fp64.
 */
int oracle_moe_ffn_mixed(const uint16_t* x, const int32_t* idx, const double* w,
                         const uint8_t* bits,
                         const uint16_t* const* w_bf16, const uint8_t* const* codes,
                         const uint16_t* const* scale, const uint16_t* const* zero,
                         int T, int H, int F, int E, int k, int group, double* y)
{
    const size_t P = (size_t)T * (size_t)k;
    double* hbuf = (double*)malloc(sizeof(double) * (P ? P : 1) * (size_t)F);
    double* obuf = (double*)malloc(sizeof(double) * (P ? P : 1) * (size_t)H);
    double* row1 = (double*)malloc(sizeof(double) * (size_t)(H > F ? H : F));
    double* row3 = (double*)malloc(sizeof(double) * (size_t)(H > F ? H : F));
    double* xd = (double*)malloc(sizeof(double) * ((size_t)T * (size_t)H + 1));
    int rc = 0;
    for (size_t i = 0; i < (size_t)T * (size_t)H; i++) xd[i] = (double)bf16_to_f32(x[i]);
    for (size_t p = 0; p < P * (size_t)H; p++) obuf[p] = 0.0;
    for (int e = 0; e < E && rc == 0; e++) {
        int b = bits[e];
        if (b == 0) continue;
        if (b != 16 && b != 8 && b != 4 && b != 2) { rc = -1; break; }
        /* pairs routed to this expert */
        size_t n_pairs = 0;
        for (size_t p = 0; p < P; p++)
            if (idx[p] == e) n_pairs++;
        if (n_pairs == 0) continue;
        const uint16_t* wb1 = w_bf16 ? w_bf16[3 * e + 0] : NULL;
        const uint16_t* wb3 = w_bf16 ? w_bf16[3 * e + 1] : NULL;
        const uint16_t* wb2 = w_bf16 ? w_bf16[3 * e + 2] : NULL;
        const uint8_t *c1 = NULL, *c3 = NULL, *c2 = NULL;
        const uint16_t *s1 = NULL, *s3 = NULL, *s2 = NULL, *z1 = NULL, *z3 = NULL, *z2 = NULL;
        if (b != 16) {
            c1 = codes[3 * e + 0]; c3 = codes[3 * e + 1]; c2 = codes[3 * e + 2];
            s1 = scale[3 * e + 0]; s3 = scale[3 * e + 1]; s2 = scale[3 * e + 2];
            z1 = zero[3 * e + 0];  z3 = zero[3 * e + 1];  z2 = zero[3 * e + 2];
            if (!c1 || !c3 || !c2 || !s1 || !s3 || !s2 || !z1 || !z3 || !z2) { rc = -2; break; }
        } else if (!wb1 || !wb3 || !wb2) { rc = -2; break; }
        for (int f = 0; f < F; f++) {
            fetch_row(b, wb1, c1, s1, z1, H, group, f, row1);
            fetch_row(b, wb3, c3, s3, z3, H, group, f, row3);
            for (size_t p = 0; p < P; p++) {
                if (idx[p] != e) continue;
                size_t t = p / (size_t)k;
                double a = 0.0, g = 0.0;
                for (int h = 0; h < H; h++) {
                    double xv = xd[t * H + h];
                    a += row1[h] * xv;
                    g += row3[h] * xv;
                }
                hbuf[p * F + f] = a / (1.0 + exp(-a)) * g;
            }
        }
        for (int j = 0; j < H; j++) {
            fetch_row(b, wb2, c2, s2, z2, F, group, j, row1);
            for (size_t p = 0; p < P; p++) {
                if (idx[p] != e) continue;
                double o = 0.0;
                for (int f = 0; f < F; f++) o += row1[f] * hbuf[p * F + f];
                obuf[p * H + j] = o;
            }
        }
    }
    if (rc == 0) {
        for (int t = 0; t < T; t++)
            for (int j = 0; j < H; j++) {
                double acc = 0.0;
                for (int s = 0; s < k; s++) {
                    size_t p = (size_t)t * k + s;
                    if (bits[idx[p]] == 0) continue;
                    acc += w[p] * obuf[p * H + j];
                }
                y[(size_t)t * H + j] = acc;
            }
    }
    free(hbuf);
    free(obuf);
    free(row1);
    free(row3);
    free(xd);
    return rc;
}

/* ------------------------------------------------------------------ */
/* Glue between the layers of an expert-only stack (not from the paper, which  */
/* runs whole transformer blocks): v = h + alpha * y, out = bf16(v / rms(v)),   */
/* in fp64, rounded once to bf16 (nearest even, through binary32).  A row of    */
/* zeros stays zero.                                                            */
/* ------------------------------------------------------------------ */

static uint16_t f64_to_bf16_rne(double d)
{
    float f = (float)d;
    uint32_t u;
    memcpy(&u, &f, sizeof u);
    u = (u + 0x7fffu + ((u >> 16) & 1u)) >> 16;
    return (uint16_t)u;
}

uint16_t oracle_f64_to_bf16(double d) { return f64_to_bf16_rne(d); }

void oracle_residual_rmsnorm(const uint16_t* h, const double* y, double alpha, int T, int H,
                             uint16_t* out)
{
    for (int t = 0; t < T; t++) {
        double ss = 0.0;
        for (int j = 0; j < H; j++) {
            double v = (double)bf16_to_f32(h[(size_t)t * H + j]) + alpha * y[(size_t)t * H + j];
            ss += v * v;
        }
        double rms = sqrt(ss / (double)H);
        for (int j = 0; j < H; j++) {
            double v = (double)bf16_to_f32(h[(size_t)t * H + j]) + alpha * y[(size_t)t * H + j];
            out[(size_t)t * H + j] = f64_to_bf16_rne(rms > 0.0 ? v / rms : 0.0);
        }
    }
}

