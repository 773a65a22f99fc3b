// Attention-derived token score (paper Sec. 4.2.1, first equation):
//   s_i = (1/Hh) sum_h a_i^(h),   a_i^(h) = (1/T) sum_q P^(h)[q, i],
// the attention token i receives, averaged over queries and heads, where
// P^(h) = softmax over keys of (q_q . k_i) * scale, keys after the query masked
// out when `causal`.  The probabilities are never stored: one pass over the keys
// gives every query's softmax maximum and normaliser, a second pass rebuilds the
// logits tile by tile and adds exp(logit - max) / normaliser into per-key sums.
//
// Both passes compute tiles of S^T = K Q^T (keys down, queries across) with
// v_mfma_f32_32x32x16_bf16.  Queries and keys are [token][head][d] rows, so a
// lane's 16-byte pieces of a row are at once the A operand (keys) and the B
// operand (queries): for short sequences nothing goes through LDS (long ones
// share the streamed operand between wavefronts, see below).  In the result a lane holds one
// query (column) and 16 keys (rows): the softmax statistics of a query and the
// running per-key sums both stay inside a lane until the very end.
#include "common.hpp"

namespace dymoe {

constexpr int kAtThreads = 256;
constexpr int kAtWaves = kAtThreads / kWave;
constexpr int kAtWideFrags = 32;       // from this many 32-token fragments on (T > 992): the LDS-staged kernels

// One lane's share of a 32-token fragment of one head (D columns): lane (ln, kb)
// holds row ln; piece c covers columns 32 (c / 2) + 16 kb + 8 (c % 2) .. + 7, i.e.
// 32 contiguous bytes per pair of pieces.  Queries and keys use the same
// column order, so the contraction is over matching columns.
template <int D>
struct AtFrag {
    uint4 c[D / 16];
};

template <int D>
__device__ __forceinline__ void load_frag(const uint16_t* __restrict__ head_base, long row_stride, int row,
                                          int kb, AtFrag<D>& f)
{
    const uint16_t* p = head_base + (long)row * row_stride + kb * 16;
#pragma unroll
    for (int c2 = 0; c2 < D / 32; c2++) {
        f.c[2 * c2] = load_global<uint4>(p + c2 * 32);
        f.c[2 * c2 + 1] = load_global<uint4>(p + c2 * 32 + 8);
    }
}

// S^T tile: rows = the 32 keys of fk, columns = the 32 queries of fq.
// Lane (ln, kb), register i: key 8 (i / 4) + 4 kb + i % 4, query ln.
template <int D>
__device__ __forceinline__ float16_t logits_tile(const AtFrag<D>& fk, const AtFrag<D>& fq)
{
    float16_t acc;
#pragma unroll
    for (int i = 0; i < 16; i++) acc[i] = 0.0f;
#pragma unroll
    for (int c = 0; c < D / 16; c++)
        acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, fk.c[c]),
                                                      __builtin_bit_cast(bf16x8_t, fq.c[c]), acc, 0, 0, 0);
    return acc;
}

__device__ __forceinline__ int tile_key(int kf, int kb, int i) { return kf * 32 + 8 * (i >> 2) + 4 * kb + (i & 3); }

// Workgroup -> (fragment, head).  Workgroups are handed to the 8 XCDs in turn
// (linear id modulo 8), each with an L2 of its own: when the heads divide
// evenly, every XCD gets whole heads, so that one head's queries and keys are
// read through one L2 instead of all eight.
__device__ __forceinline__ void fragment_and_head(int nfrag, int n_heads, int& frag, int& head)
{
    const int lin = blockIdx.x + gridDim.x * blockIdx.y;      // grid = (nfrag, n_heads)
    if (n_heads % 8 == 0) {
        const int xcd = lin & 7, j = lin >> 3, per = n_heads >> 3;
        head = xcd * per + j / nfrag;
        frag = j - (j / nfrag) * nfrag;
    } else {
        frag = blockIdx.x;
        head = blockIdx.y;
    }
}

constexpr float kMasked = -1.0e30f;     // finite stand-in for minus infinity: no NaN from (-inf) - (-inf)

// Pass 1.  A workgroup owns 32 queries of one head; its four wavefronts take
// every fourth key fragment each (interleaved, so a causal mask leaves them
// equal shares) and keep a running maximum m and sum l of exp2(logit' - m),
// logit' = logit * scale * log2(e); the four (m, l) pairs of a query are merged
// through LDS in wavefront order.  stats[h][q] = (m, 1 / l).
template <int D>
__global__ __launch_bounds__(kAtThreads) void attn_rowstats_kernel(
    const uint16_t* __restrict__ q, const uint16_t* __restrict__ k, int T, int n_heads, int group,
    float scale_log2, int causal, float2* __restrict__ stats)
{
    __shared__ float2 s_ml[kAtWaves][32];
    const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
    const int ln = lane & 31, kb = lane >> 5;
    const int nfrag = (T + 31) >> 5;
    int qf, h;
    fragment_and_head(nfrag, n_heads, qf, h);
    const long q_stride = (long)n_heads * D, k_stride = (long)(n_heads / group) * D;
    const uint16_t* qh = q + (long)h * D;
    const uint16_t* kh = k + (long)(h / group) * D;
    const int query = qf * 32 + ln;
    AtFrag<D> fq, fk, fn;
    load_frag<D>(qh, q_stride, min(query, T - 1), kb, fq);     // rows past the end re-read the last token; masked below
    const int kf_last = causal ? qf : nfrag - 1;
    load_frag<D>(kh, k_stride, min(wave * 32 + ln, T - 1), kb, fk);
    float m = kMasked, l = 0.0f;
    for (int kf = wave; kf <= kf_last; kf += kAtWaves) {
        const int kn = (kf + kAtWaves <= kf_last) ? kf + kAtWaves : kf;   // the next fragment is requested before this one is used
        load_frag<D>(kh, k_stride, min(kn * 32 + ln, T - 1), kb, fn);
        const float16_t acc = logits_tile<D>(fk, fq);
        float sv[16];
        float mx = m;
#pragma unroll
        for (int i = 0; i < 16; i++) {
            const int key = tile_key(kf, kb, i);
            const bool ok = key < T && (!causal || key <= query);
            sv[i] = ok ? acc[i] * scale_log2 : kMasked;
            mx = fmaxf(mx, sv[i]);
        }
        float add = 0.0f;
#pragma unroll
        for (int i = 0; i < 16; i++) add += (sv[i] > 0.5f * kMasked) ? __builtin_amdgcn_exp2f(sv[i] - mx) : 0.0f;
        l = l * __builtin_amdgcn_exp2f(m - mx) + add;
        m = mx;
        fk = fn;
    }
    // the two halves of the keys (kb = 0, 1) of this query
    const float m2 = __shfl_xor(m, 32, kWave), l2 = __shfl_xor(l, 32, kWave);
    float M = fmaxf(m, m2);
    float L = l * __builtin_amdgcn_exp2f(m - M) + l2 * __builtin_amdgcn_exp2f(m2 - M);
    if (kb == 0) s_ml[wave][ln] = make_float2(M, L);
    __syncthreads();
    if (wave == 0 && kb == 0 && query < T) {
        M = s_ml[0][ln].x;
#pragma unroll
        for (int w = 1; w < kAtWaves; w++) M = fmaxf(M, s_ml[w][ln].x);
        L = 0.0f;
#pragma unroll
        for (int w = 0; w < kAtWaves; w++) L += s_ml[w][ln].y * __builtin_amdgcn_exp2f(s_ml[w][ln].x - M);
        stats[(long)h * T + query] = make_float2(M, 1.0f / L);
    }
}

// Pass 2.  A workgroup owns 32 keys of one head; its wavefronts take every fourth
// query fragment among those that see the keys:
// partial[h][key] = sum_q exp2(logit' - m_q) / l_q, the four wavefronts' sums added in order.
template <int D>
__global__ __launch_bounds__(kAtThreads) void attn_colsum_kernel(
    const uint16_t* __restrict__ q, const uint16_t* __restrict__ k, int T, int n_heads, int group,
    float scale_log2, int causal, const float2* __restrict__ stats, float* __restrict__ partial)
{
    __shared__ float s_col[kAtWaves][32];
    const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
    const int ln = lane & 31, kb = lane >> 5;
    const int nfrag = (T + 31) >> 5;
    int kf, h;
    fragment_and_head(nfrag, n_heads, kf, h);
    const long q_stride = (long)n_heads * D, k_stride = (long)(n_heads / group) * D;
    const uint16_t* qh = q + (long)h * D;
    const uint16_t* kh = k + (long)(h / group) * D;
    const float2* sh = stats + (long)h * T;
    AtFrag<D> fk, fq, fn;
    load_frag<D>(kh, k_stride, min(kf * 32 + ln, T - 1), kb, fk);
    const int qf_first = (causal ? kf : 0) + wave;
    load_frag<D>(qh, q_stride, min(qf_first * 32 + ln, T - 1), kb, fq);
    float2 st = sh[min(qf_first * 32 + ln, T - 1)];
    float col[16];
#pragma unroll
    for (int i = 0; i < 16; i++) col[i] = 0.0f;
    for (int qf = qf_first; qf < nfrag; qf += kAtWaves) {
        const int qn = (qf + kAtWaves < nfrag) ? qf + kAtWaves : qf;
        load_frag<D>(qh, q_stride, min(qn * 32 + ln, T - 1), kb, fn);
        const float2 stn = sh[min(qn * 32 + ln, T - 1)];
        const float16_t acc = logits_tile<D>(fk, fq);
        const int query = qf * 32 + ln;
#pragma unroll
        for (int i = 0; i < 16; i++) {
            const int key = tile_key(kf, kb, i);
            const bool ok = query < T && key < T && (!causal || key <= query);
            const float p = __builtin_amdgcn_exp2f(acc[i] * scale_log2 - st.x) * st.y;
            col[i] += ok ? p : 0.0f;
        }
        fq = fn;
        st = stn;
    }
    // sum over the 32 queries held by the lanes of each half
#pragma unroll
    for (int i = 0; i < 16; i++) {
        float v = col[i];
#pragma unroll
        for (int o = 16; o > 0; o >>= 1) v += __shfl_xor(v, o, kWave);
        col[i] = v;
    }
    if (ln == 0) {
#pragma unroll
        for (int i = 0; i < 16; i++) s_col[wave][tile_key(0, kb, i)] = col[i];
    }
    __syncthreads();
    if (threadIdx.x < 32) {
        const int key = kf * 32 + threadIdx.x;
        float v = s_col[0][threadIdx.x];
#pragma unroll
        for (int w = 1; w < kAtWaves; w++) v += s_col[w][threadIdx.x];
        if (key < T) partial[(long)h * T + key] = v;
    }
}

// ----------------------------------------------------------------------------
// Long sequences: the streamed operand goes through LDS.  A workgroup owns 128
// tokens (one 32-token fragment per wavefront, kept in registers) and all four
// wavefronts multiply against the same streamed fragment, which the workgroup
// fetches once with whole-row coalesced loads and parks in LDS (two buffers;
// 16-byte chunk c of row r at chunk position c ^ (r mod chunks-per-row), so that
// the operand reads of 16 consecutive rows fall on different banks).  A quarter
// of the global traffic of the short-sequence kernels, and no merge between
// wavefronts: each owns its tokens' statistics or sums outright.
template <int D>
struct AtStage {
    static constexpr int kPerThread = 32 * (D / 8) / kAtThreads;      // 2 (D = 128) or 1 (D = 64)
    uint4 v[kPerThread];
};

template <int D>
__device__ __forceinline__ void stage_fetch(const uint16_t* __restrict__ head_base, long row_stride, int row0, int T,
                                            AtStage<D>& st)
{
    constexpr int CH = D / 8;
#pragma unroll
    for (int i = 0; i < AtStage<D>::kPerThread; i++) {
        const int at = i * kAtThreads + threadIdx.x;
        const int r = at / CH, c = at % CH;
        st.v[i] = load_global<uint4>(head_base + (long)min(row0 + r, T - 1) * row_stride + c * 8);
    }
}

template <int D>
__device__ __forceinline__ void stage_store(char* buf, const AtStage<D>& st)
{
    constexpr int CH = D / 8;
#pragma unroll
    for (int i = 0; i < AtStage<D>::kPerThread; i++) {
        const int at = i * kAtThreads + threadIdx.x;
        const int r = at / CH, c = at % CH;
        *reinterpret_cast<uint4*>(buf + r * (D * 2) + ((c ^ (r & (CH - 1))) << 4)) = st.v[i];
    }
}

// the lane's share of the staged fragment, in the piece order of load_frag
template <int D>
__device__ __forceinline__ void frag_from_lds(const char* buf, int ln, int kb, AtFrag<D>& f)
{
    constexpr int CH = D / 8;
#pragma unroll
    for (int c = 0; c < D / 16; c++) {
        const int ch = (c >> 1) * 4 + kb * 2 + (c & 1);
        f.c[c] = *reinterpret_cast<const uint4*>(buf + ln * (D * 2) + ((ch ^ (ln & (CH - 1))) << 4));
    }
}

// Pass 1, long sequences: wavefront w owns queries 128 blk + 32 w .. + 31; keys stream through LDS.
template <int D>
__global__ __launch_bounds__(kAtThreads) void attn_rowstats_wide_kernel(
    const uint16_t* __restrict__ q, const uint16_t* __restrict__ k, int T, int n_heads, int group,
    float scale_log2, int causal, float2* __restrict__ stats)
{
    __shared__ __attribute__((aligned(16))) char s_buf[2][32 * D * 2];
    const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
    const int ln = lane & 31, kb = lane >> 5;
    const int nfrag = (T + 31) >> 5;
    int blk, h;
    fragment_and_head((nfrag + 3) >> 2, n_heads, blk, h);
    const long q_stride = (long)n_heads * D, k_stride = (long)(n_heads / group) * D;
    const uint16_t* qh = q + (long)h * D;
    const uint16_t* kh = k + (long)(h / group) * D;
    const int qf = 4 * blk + wave;
    const int query = qf * 32 + ln;
    AtFrag<D> fq, fk;
    load_frag<D>(qh, q_stride, min(query, T - 1), kb, fq);
    const int kf_last = causal ? min(4 * blk + 3, nfrag - 1) : nfrag - 1;
    AtStage<D> st;
    stage_fetch<D>(kh, k_stride, 0, T, st);
    stage_store<D>(s_buf[0], st);
    __syncthreads();
    float m = kMasked, l = 0.0f;
    for (int kf = 0; kf <= kf_last; kf++) {
        const bool more = kf < kf_last;                         // the same in every thread
        if (more) stage_fetch<D>(kh, k_stride, (kf + 1) * 32, T, st);
        if (qf < nfrag && (!causal || kf <= qf)) {              // the same in every lane of the wavefront
            frag_from_lds<D>(s_buf[kf & 1], ln, kb, fk);
            const float16_t acc = logits_tile<D>(fk, fq);
            if (kf * 32 + 31 < T && (!causal || kf < qf)) {
                // nothing to mask (the rule for all but the diagonal and the last fragment): the scale is positive,
                // so the maximum is taken over the raw logits and the scale rides in the exponent's multiply-add
                float raw = acc[0];
#pragma unroll
                for (int i = 1; i < 16; i++) raw = fmaxf(raw, acc[i]);
                const float mx = fmaxf(m, raw * scale_log2);
                float add = 0.0f;
#pragma unroll
                for (int i = 0; i < 16; i++) add += __builtin_amdgcn_exp2f(fmaf(acc[i], scale_log2, -mx));
                l = l * __builtin_amdgcn_exp2f(m - mx) + add;
                m = mx;
            } else {
                float sv[16];
                float mx = m;
#pragma unroll
                for (int i = 0; i < 16; i++) {
                    const int key = tile_key(kf, kb, i);
                    const bool ok = key < T && (!causal || key <= query);
                    sv[i] = ok ? acc[i] * scale_log2 : kMasked;
                    mx = fmaxf(mx, sv[i]);
                }
                float add = 0.0f;
#pragma unroll
                for (int i = 0; i < 16; i++) add += (sv[i] > 0.5f * kMasked) ? __builtin_amdgcn_exp2f(sv[i] - mx) : 0.0f;
                l = l * __builtin_amdgcn_exp2f(m - mx) + add;
                m = mx;
            }
        }
        if (more) stage_store<D>(s_buf[(kf + 1) & 1], st);
        __syncthreads();
    }
    const float m2 = __shfl_xor(m, 32, kWave), l2 = __shfl_xor(l, 32, kWave);
    const float M = fmaxf(m, m2);
    const float L = l * __builtin_amdgcn_exp2f(m - M) + l2 * __builtin_amdgcn_exp2f(m2 - M);
    // one number per query is all pass 2 needs: p = exp2(logit' - (m + log2 l))
    if (kb == 0 && query < T) stats[(long)h * T + query] = make_float2(M + __builtin_amdgcn_logf(L), 0.0f);
}

// Pass 2, long sequences: wavefront w owns keys 128 blk + 32 w .. + 31; queries stream through LDS.
template <int D>
__global__ __launch_bounds__(kAtThreads) void attn_colsum_wide_kernel(
    const uint16_t* __restrict__ q, const uint16_t* __restrict__ k, int T, int n_heads, int group,
    float scale_log2, int causal, const float2* __restrict__ stats, float* __restrict__ partial)
{
    __shared__ __attribute__((aligned(16))) char s_buf[2][32 * D * 2];
    const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
    const int ln = lane & 31, kb = lane >> 5;
    const int nfrag = (T + 31) >> 5;
    int blk, h;
    fragment_and_head((nfrag + 3) >> 2, n_heads, blk, h);
    const long q_stride = (long)n_heads * D, k_stride = (long)(n_heads / group) * D;
    const uint16_t* qh = q + (long)h * D;
    const uint16_t* kh = k + (long)(h / group) * D;
    const float2* sh = stats + (long)h * T;
    const int kf = 4 * blk + wave;
    AtFrag<D> fk, fq;
    load_frag<D>(kh, k_stride, min(kf * 32 + ln, T - 1), kb, fk);
    const int qf_first = causal ? 4 * blk : 0;
    AtStage<D> st;
    stage_fetch<D>(qh, q_stride, qf_first * 32, T, st);
    stage_store<D>(s_buf[0], st);
    __syncthreads();
    float col[16];
#pragma unroll
    for (int i = 0; i < 16; i++) col[i] = 0.0f;
    for (int qf = qf_first; qf < nfrag; qf++) {
        const bool more = qf + 1 < nfrag;
        if (more) stage_fetch<D>(qh, q_stride, (qf + 1) * 32, T, st);
        if (kf < nfrag && (!causal || qf >= kf)) {
            const int query = qf * 32 + ln;
            const float shift = -sh[min(query, T - 1)].x;
            frag_from_lds<D>(s_buf[(qf - qf_first) & 1], ln, kb, fq);
            const float16_t acc = logits_tile<D>(fk, fq);
            if (qf * 32 + 31 < T && kf * 32 + 31 < T && (!causal || kf < qf)) {
#pragma unroll
                for (int i = 0; i < 16; i++) col[i] += __builtin_amdgcn_exp2f(fmaf(acc[i], scale_log2, shift));
            } else {
#pragma unroll
                for (int i = 0; i < 16; i++) {
                    const int key = tile_key(kf, kb, i);
                    const bool ok = query < T && key < T && (!causal || key <= query);
                    const float p = __builtin_amdgcn_exp2f(fmaf(acc[i], scale_log2, shift));
                    col[i] += ok ? p : 0.0f;
                }
            }
        }
        if (more) stage_store<D>(s_buf[(qf + 1 - qf_first) & 1], st);
        __syncthreads();
    }
#pragma unroll
    for (int i = 0; i < 16; i++) {
        float v = col[i];
#pragma unroll
        for (int o = 16; o > 0; o >>= 1) v += __shfl_xor(v, o, kWave);
        col[i] = v;
    }
    if (ln == 0 && kf < nfrag) {
#pragma unroll
        for (int i = 0; i < 16; i++) {
            const int key = tile_key(kf, kb, i);
            if (key < T) partial[(long)h * T + key] = col[i];
        }
    }
}

// s[i] = (sum over heads, in head order) / (Hh T)
__global__ __launch_bounds__(256) void attn_score_kernel(const float* __restrict__ partial, int T, int n_heads,
                                                         float inv, float* __restrict__ score)
{
    const int i = blockIdx.x * 256 + threadIdx.x;
    if (i >= T) return;
    float s = 0.0f;
    for (int h = 0; h < n_heads; h++) s += partial[(long)h * T + i];
    score[i] = s * inv;
}

static size_t attn_stats_bytes(int T, int n_heads) { return ((size_t)T * n_heads * sizeof(float2) + 255) / 256 * 256; }

}  // namespace dymoe

extern "C" {

size_t dymoe_attention_workspace_bytes(int T, int n_heads)
{
    if (T <= 0 || n_heads <= 0) return 0;
    return dymoe::attn_stats_bytes(T, n_heads) + ((size_t)T * n_heads * sizeof(float) + 255) / 256 * 256;
}

int dymoe_token_score_attention(dymoe_ctx* ctx, const void* q, const void* k, int T, int n_heads,
                                int n_kv_heads, int head_dim, float scale, int causal, float* score,
                                void* workspace, size_t workspace_bytes, void* stream)
{
    DYMOE_REQUIRE(T >= 0 && n_heads > 0 && n_kv_heads > 0 && n_heads % n_kv_heads == 0);
    DYMOE_REQUIRE(head_dim > 0 && head_dim % 8 == 0);
    DYMOE_REQUIRE(scale >= 0.0f && (causal == 0 || causal == 1));
    if (T == 0) return ctx ? DYMOE_OK : DYMOE_ENOCTX;
    DYMOE_REQUIRE(q && k && score && workspace);
    DYMOE_REQUIRE(dymoe_aligned(q, 16) && dymoe_aligned(k, 16) && dymoe_aligned(score, 4) &&
                  dymoe_aligned(workspace, 256));
    if (head_dim != 64 && head_dim != 128) return DYMOE_ENOTSUP;
    if (n_heads > 65535) return DYMOE_ENOTSUP;
    if (workspace_bytes < dymoe_attention_workspace_bytes(T, n_heads)) return DYMOE_ENOSPC;
    if (!ctx) return DYMOE_ENOCTX;
    hipStream_t st = (hipStream_t)stream;
    const uint16_t* qb = (const uint16_t*)q;
    const uint16_t* kbp = (const uint16_t*)k;
    float2* stats = reinterpret_cast<float2*>(workspace);
    float* partial = reinterpret_cast<float*>((char*)workspace + dymoe::attn_stats_bytes(T, n_heads));
    const int group = n_heads / n_kv_heads;
    const float s = (scale > 0.0f) ? scale : 1.0f / sqrtf((float)head_dim);
    const float scale_log2 = s * 1.44269504088896340736f;
    const int nfrag = (T + 31) / 32;
    // short sequences: a workgroup per 32-token fragment (many workgroups, operands straight from global memory);
    // long ones: a workgroup per 128 tokens with the streamed operand shared through LDS
    const bool wide = nfrag >= dymoe::kAtWideFrags;
    const dim3 grid((unsigned)(wide ? (nfrag + 3) / 4 : nfrag), (unsigned)n_heads);
#define DYMOE_ATTN_LAUNCH(D_)                                                                                          \
    do {                                                                                                               \
        if (wide) {                                                                                                    \
            dymoe_launch(ctx, DYMOE_K_ATTN_STATS, dymoe::attn_rowstats_wide_kernel<D_>, grid, dim3(dymoe::kAtThreads), 0, st, \
                         qb, kbp, T, n_heads, group, scale_log2, causal, stats);                                       \
            DYMOE_HIP_LAUNCH_CHECK();                                                                                  \
            dymoe_launch(ctx, DYMOE_K_ATTN_COLSUM, dymoe::attn_colsum_wide_kernel<D_>, grid, dim3(dymoe::kAtThreads), 0, st, \
                         qb, kbp, T, n_heads, group, scale_log2, causal, (const float2*)stats, partial);               \
        } else {                                                                                                       \
            dymoe_launch(ctx, DYMOE_K_ATTN_STATS, dymoe::attn_rowstats_kernel<D_>, grid, dim3(dymoe::kAtThreads), 0, st,  \
                         qb, kbp, T, n_heads, group, scale_log2, causal, stats);                                       \
            DYMOE_HIP_LAUNCH_CHECK();                                                                                  \
            dymoe_launch(ctx, DYMOE_K_ATTN_COLSUM, dymoe::attn_colsum_kernel<D_>, grid, dim3(dymoe::kAtThreads), 0, st,   \
                         qb, kbp, T, n_heads, group, scale_log2, causal, (const float2*)stats, partial);               \
        }                                                                                                              \
    } while (0)
    if (head_dim == 64) DYMOE_ATTN_LAUNCH(64);
    else DYMOE_ATTN_LAUNCH(128);
#undef DYMOE_ATTN_LAUNCH
    DYMOE_HIP_LAUNCH_CHECK();
    hipLaunchKernelGGL(dymoe::attn_score_kernel, dim3((unsigned)((T + 255) / 256)), dim3(256), 0, st,
                       (const float*)partial, T, n_heads, 1.0f / ((float)n_heads * (float)T), score);
    DYMOE_HIP_LAUNCH_CHECK();
    return DYMOE_OK;
}

}  // extern "C"
