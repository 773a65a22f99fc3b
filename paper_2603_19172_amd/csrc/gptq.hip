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
// Rows are independent, columns are not.  Per group of 64 columns two kinds of launch:
//   group kernel   a lane owns a row: the group's 64 values in registers, the
//                  64 x 64 diagonal block of U staged in LDS and read as
//                  broadcasts (every lane needs the same value); quantises the 64 columns
//                  in order, applies the corrections inside the group, writes
//                  codes, scale, zero and the 64 errors e of the row;
//   trail kernel   v[:, j] for later columns j: 64 chained FMAs per element and
//                  group, a workgroup on a 64-row x 128-column tile with the
//                  errors and the 64 x 128 block of U in LDS, 8 x 4 elements per
//                  thread.  Groups go in pairs: the first group's corrections
//                  reach the second group's columns at once, and both groups'
//                  128 corrections then go over the remaining columns in one pass.
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

// One group of 64 columns for the rows [row_begin, row_end), a lane per row.
//   BITS = 2, 4, 8   the quantizer: codes, scale and zero of the group are written, e is the scaled rounding error;
//   BITS = 0         nothing is quantised and e = x[c] / D[c,c]: the row is solved against the upper triangular
//                    diagonal block D (forward substitution; the factorisation below is built from this).
// x: the rows' current values of the group's columns, x[row * ldx + c]; d: the 64 x 64 diagonal block, d[c * ldd + j].
// e of (column c, row) goes to own_p[c * own_cs + row * own_rs] (OWN; the row range must then be whole blocks of 64)
// and to pad_p[c * pad_cs + slot * pad_rs] (PAD) for every lane of the grid, rows rounded up to 64: a buffer of that
// many rows, from which the trail kernel loads whole 64-row tiles.  Which of the two are written is fixed at compile
// time: with run-time tests around the stores the 64 unrolled columns fall apart into basic blocks, and the
// values the compiler keeps across them spill.
template <int BITS, bool OWN, bool PAD>
__global__ __launch_bounds__(kGqRows) void gptq_group_kernel(
    const float* __restrict__ x_in, long ldx, const float* __restrict__ d, long ldd, long row_begin, long row_end,
    float* __restrict__ own_p, long own_cs, long own_rs, float* __restrict__ pad_p, long pad_cs, long pad_rs,
    uint8_t* __restrict__ codes, uint16_t* __restrict__ scale, uint16_t* __restrict__ zero,
    long code_row_bytes, long groups_per_row)
{
#pragma clang fp contract(off)
    const long slot = row_begin + (long)blockIdx.x * kGqRows + threadIdx.x;
    const bool mine = slot < row_end;
    const long row = min(slot, row_end - 1);        // lanes past the last row redo it and keep the result to themselves
    float x[kGqGroup];
#pragma unroll
    for (int c = 0; c < kGqGroup / 4; c++) {
        const float4 q = *reinterpret_cast<const float4*>(x_in + row * ldx + 4 * c);
        x[4 * c + 0] = q.x; x[4 * c + 1] = q.y; x[4 * c + 2] = q.z; x[4 * c + 3] = q.w;
    }
    constexpr int qmax = BITS ? (1 << BITS) - 1 : 1;
    constexpr int per_word = BITS ? 32 / BITS : 32;
    constexpr int n_words = BITS ? kGqGroup / per_word : 1;   // 16 (int8), 8 (int4), 4 (int2)
    float m = 0.0f, s = 0.0f, inv = 0.0f;
    _Float16 zh = (_Float16)0.0f, sh = (_Float16)0.0f;
    if constexpr (BITS != 0) {
        float lo = x[0], hi = x[0];
#pragma unroll
        for (int i = 1; i < kGqGroup; i++) {
            lo = fminf(lo, x[i]);
            hi = fmaxf(hi, x[i]);
        }
        zh = (_Float16)lo;                          // round to nearest even
        const float range = hi - lo;
        const float step = range / (float)qmax;     // correctly rounded division
        sh = (_Float16)step;
        m = (float)zh;
        s = (float)sh;
        inv = (s > 0.0f) ? (1.0f / s) : 0.0f;
    }
    // The diagonal block goes through LDS: every lane needs every value, one row per column step, and fetched row
    // by row from memory (the scalar cache's way) each step would wait out a full memory latency: 64 in a chain.
    __shared__ __attribute__((aligned(16))) float s_d[kGqGroup][kGqGroup + 4];   // + 4: the row-per-lane staging stores spread over the banks
#pragma unroll
    for (int c = 0; c < kGqGroup / 4; c++)
        *reinterpret_cast<float4*>(&s_d[threadIdx.x][4 * c]) =
            *reinterpret_cast<const float4*>(d + (long)threadIdx.x * ldd + 4 * c);
    __syncthreads();
    uint32_t words[n_words];
#pragma unroll
    for (int i = 0; i < n_words; i++) words[i] = 0u;
#pragma unroll
    for (int i = 0; i < kGqGroup; i++) {
        float rest = x[i];
        if constexpr (BITS != 0) {
            const float t = x[i] - m;
            float r = __builtin_rintf(t * inv);
            r = fminf(fmaxf(r, 0.0f), (float)qmax);
            words[i / per_word] |= (uint32_t)(int)r << (BITS * (i % per_word));
            float dq = r * s;
            dq = dq + m;
            rest = x[i] - dq;
        }
        const float e = rest / s_d[i][i];
        if constexpr (OWN) own_p[(long)i * own_cs + slot * own_rs] = e;
        if constexpr (PAD) pad_p[(long)i * pad_cs + slot * pad_rs] = e;
        const float ne = -e;
#pragma unroll
        for (int j = i + 1; j < kGqGroup; j++) x[j] = __builtin_fmaf(ne, s_d[i][j], x[j]);
    }
    if constexpr (BITS != 0) {
        if (mine) {
            uint8_t* dst = codes + row * code_row_bytes;
#pragma unroll
            for (int i = 0; i < n_words / 4; i++)
                store_global(dst + 16 * i, make_uint4(words[4 * i], words[4 * i + 1], words[4 * i + 2], words[4 * i + 3]));
            store_global(scale + row * groups_per_row, (uint16_t)f16_bits(sh));
            store_global(zero + row * groups_per_row, (uint16_t)f16_bits(zh));
        }
    }
}

// v[r, j] = fma(-E[c, r], B[c, j], v[r, j]) for c = 0 .. 64 n_chunks - 1 in that order (one or two groups' worth of
// corrections in one pass over v: the working copy is what this kernel streams), rows [row_begin, row_end) in tiles of
// 64 from row_begin, columns [col_begin, col_end) in tiles of 128 from col_begin.  E[c, r] = e[c * lde + r] (whole
// 64-row tiles are loaded: the buffer covers the rows rounded up), B[c, j] = b[c * ldb + j].  lower_only: tiles that
// lie wholly above the diagonal (every row < every column) are left alone.
__global__ __launch_bounds__(kGqTrailThreads) void gptq_trail_kernel(
    float* __restrict__ v, long ldv, const float* __restrict__ e, long lde, const float* __restrict__ b, long ldb,
    long row_begin, long row_end, long col_begin, long col_end, int n_chunks, int lower_only)
{
    __shared__ __attribute__((aligned(16))) float s_e[kGqGroup][kGqRows];
    __shared__ __attribute__((aligned(16))) float s_u[kGqGroup][kGqTrailCols];
    const int tid = threadIdx.x;
    const long col0 = col_begin + (long)blockIdx.x * kGqTrailCols;
    const long row0 = row_begin + (long)blockIdx.y * kGqRows;
    if (lower_only && row0 + kGqRows - 1 < col0) return;        // the whole workgroup
    const int tx = tid & 31, ty = tid >> 5;
    const long col = col0 + 4 * tx;
    const long row = row0 + 8 * ty;
    const bool in_cols = col < col_end;
    float4 acc[8];
#pragma unroll
    for (int i = 0; i < 8; i++) {
        acc[i] = make_float4(0.f, 0.f, 0.f, 0.f);
        if (in_cols && row + i < row_end) acc[i] = *reinterpret_cast<const float4*>(v + (row + i) * ldv + col);
    }
    for (int ch = 0; ch < n_chunks; ch++) {
        if (ch) __syncthreads();                    // the previous chunk's reads of LDS are done
        const float* ec = e + (long)ch * kGqGroup * lde;
        const float* bc = b + (long)ch * kGqGroup * ldb;
#pragma unroll
        for (int i = 0; i < kGqGroup * kGqRows / 4 / kGqTrailThreads; i++) {
            const int at = (i * kGqTrailThreads + tid) * 4;
            const int c = at / kGqRows, r = at % kGqRows;
            *reinterpret_cast<float4*>(&s_e[c][r]) = *reinterpret_cast<const float4*>(ec + (long)c * lde + row0 + r);
        }
#pragma unroll
        for (int i = 0; i < kGqGroup * kGqTrailCols / 4 / kGqTrailThreads; i++) {
            const int at = (i * kGqTrailThreads + tid) * 4;
            const int c = at / kGqTrailCols, n = at % kGqTrailCols;
            float4 q = make_float4(0.f, 0.f, 0.f, 0.f);
            if (col0 + n < col_end) q = *reinterpret_cast<const float4*>(bc + (long)c * ldb + col0 + n);
            *reinterpret_cast<float4*>(&s_u[c][n]) = q;
        }
        __syncthreads();
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
    }
#pragma unroll
    for (int i = 0; i < 8; i++)
        if (in_cols && row + i < row_end) *reinterpret_cast<float4*>(v + (row + i) * ldv + col) = acc[i];
}

// ---------------------------------------------------------------------------
// Hessian of the calibration inputs: hess (+)= X^T X, x [n, K] bf16, fp32 sums on the matrix cores
// (v_mfma_f32_32x32x16_bf16: the products of bf16 numbers are exact in fp32).  Both operands of a tile are
// columns of X, which memory holds row by row: a thread fetches an 8-sample x 8-column block with eight
// 16-byte loads, transposes it in registers and parks eight 16-byte pieces (one column, 8 samples) in LDS,
// chunk position XOR-swizzled by column so that neither the operand reads nor the transposed stores
// collide on banks.  A workgroup owns a 128 x 128 tile on or above the diagonal (64 x 64 per wavefront) and writes the
// mirror image as well.
constexpr int kHsTile = 128;
// Chunk position of column c's 16-byte pieces in LDS: a column is 128 bytes (all 32 banks), so the bank of a
// piece is its chunk position alone.  Eight neighbouring lanes must land on eight positions both when the
// operands are read (lanes = 8 consecutive columns, one chunk) and when the transposed blocks are stored
// (lanes = the same column-in-block of 8 consecutive blocks, one chunk): hence both the low bits and the
// block bits of the column go into the XOR.
__device__ __forceinline__ int hs_swizzle(int c) { return (c ^ (c >> 3)) & 7; }
constexpr int kHsSamples = 64;
constexpr int kHsThreads = 256;

__global__ __launch_bounds__(kHsThreads) void gptq_hessian_kernel(const uint16_t* __restrict__ x, long n, long K,
                                                                 int accumulate, float* __restrict__ hess)
{
    __shared__ uint4 s_op[2][kHsTile * (kHsSamples / 8)];      // [operand][column][chunk of 8 samples]
    const int tid = threadIdx.x;
    const int lane = tid & (kWave - 1), wave = tid / kWave;
    const int ln = lane & 31, kb = lane >> 5;
    // block -> tile (ti, tj), tj >= ti, rows of the upper triangle one after the other
    const int nt = (int)((K + kHsTile - 1) / kHsTile);
    int ti = 0, left = (int)blockIdx.x;
    while (left >= nt - ti) {
        left -= nt - ti;
        ti++;
    }
    const int tj = ti + left;
    const long i0 = (long)ti * kHsTile, j0 = (long)tj * kHsTile;
    // loading role: threads 0..127 the row operand's columns, 128..255 the column operand's
    const int op = tid >> 7;
    const int blk = tid & 127;
    const int sgrp = blk >> 4;                      // which 8 samples of the step's 64
    const int cgrp = blk & 15;                      // which 8 columns of the tile's 128
    const long lcol = (op ? j0 : i0) + 8 * cgrp;
    const int wi = wave >> 1, wj = wave & 1;
    float16_t acc[2][2];
#pragma unroll
    for (int a = 0; a < 2; a++)
#pragma unroll
        for (int b = 0; b < 2; b++)
#pragma unroll
            for (int i = 0; i < 16; i++) acc[a][b][i] = 0.0f;
    uint4 raw[8];
    auto fetch = [&](long s0) {
#pragma unroll
        for (int r = 0; r < 8; r++) {
            const long smp = s0 + 8 * sgrp + r;
            raw[r] = make_uint4(0u, 0u, 0u, 0u);
            if (smp < n && lcol < K) raw[r] = load_global<uint4>(x + smp * K + lcol);
        }
    };
    fetch(0);
    for (long s0 = 0; s0 < n; s0 += kHsSamples) {
        // 8 x 8 transpose of 16-bit values: pair up the rows, split even and odd columns
        uint4 out[8];
#pragma unroll
        for (int dw = 0; dw < 4; dw++) {
            uint32_t even[4], odd[4];
#pragma unroll
            for (int pr = 0; pr < 4; pr++) {
                const uint32_t a = reinterpret_cast<const uint32_t*>(&raw[2 * pr])[dw];
                const uint32_t b = reinterpret_cast<const uint32_t*>(&raw[2 * pr + 1])[dw];
                even[pr] = (a & 0xffffu) | (b << 16);
                odd[pr] = (a >> 16) | (b & 0xffff0000u);
            }
            out[2 * dw] = make_uint4(even[0], even[1], even[2], even[3]);
            out[2 * dw + 1] = make_uint4(odd[0], odd[1], odd[2], odd[3]);
        }
        __syncthreads();                            // the previous step's operand reads are done
#pragma unroll
        for (int i = 0; i < 8; i++) {
            const int c = 8 * cgrp + i;
            s_op[op][c * (kHsSamples / 8) + (sgrp ^ hs_swizzle(c))] = out[i];
        }
        __syncthreads();
        if (s0 + kHsSamples < n) fetch(s0 + kHsSamples);          // in flight during the products
#pragma unroll
        for (int ks = 0; ks < kHsSamples / 16; ks++) {
            const int chunk = 2 * ks + kb;
            bf16x8_t fa[2], fb[2];
#pragma unroll
            for (int h = 0; h < 2; h++) {
                const int ca = 64 * wi + 32 * h + ln, cb = 64 * wj + 32 * h + ln;
                fa[h] = __builtin_bit_cast(bf16x8_t, s_op[0][ca * (kHsSamples / 8) + (chunk ^ hs_swizzle(ca))]);
                fb[h] = __builtin_bit_cast(bf16x8_t, s_op[1][cb * (kHsSamples / 8) + (chunk ^ hs_swizzle(cb))]);
            }
#pragma unroll
            for (int a = 0; a < 2; a++)
#pragma unroll
                for (int b = 0; b < 2; b++)
                    acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[a], fb[b], acc[a][b], 0, 0, 0);
        }
    }
    // register i of lane (ln, kb): row 8 (i / 4) + 4 kb + i % 4 of the 32 x 32 tile, column ln
#pragma unroll
    for (int a = 0; a < 2; a++)
#pragma unroll
        for (int b = 0; b < 2; b++)
#pragma unroll
            for (int i = 0; i < 16; i++) {
                const long r = i0 + 64 * wi + 32 * a + 8 * (i >> 2) + 4 * kb + (i & 3);
                const long c = j0 + 64 * wj + 32 * b + ln;
                if (r < K && c < K) {
                    float val = acc[a][b][i];
                    if (accumulate) val += hess[r * K + c];
                    hess[r * K + c] = val;
                    if (ti != tj) hess[c * K + r] = val;
                }
            }
}

// ---------------------------------------------------------------------------
// Factor of the inverse Hessian: U upper triangular, (H + damping)^-1 = U^T U.
// With J the order-reversing permutation and J (H + damping) J = R^T R (R upper triangular, plain Cholesky),
// U = J R^-T J.  Both steps are built from the two kernels above:
//   Cholesky, per block of 64 columns: the 64 x 64 diagonal block is factored by one wavefront; the rows
//     below it are solved against that block (group kernel without quantisation: e = the new column block of
//     L = R^T, stored as rows of R); the rest of the lower triangle loses L_panel L_panel^T (trail kernel with
//     the panel, read from R, on both sides);
//   inverse: the rows of R^-T come from forward substitution of the unit vectors against R, which is the
//     quantizer's sweep with nothing quantised and the identity as the matrix; a row c only starts at its own
//     column, so a step touches rows [0, base + 64) only.  e is written straight to U's mirrored position.

// damping = damp * mean of the diagonal, a zero diagonal entry counting as (and becoming) 1
__global__ __launch_bounds__(256) void gptq_damping_kernel(const float* __restrict__ hess, long K, float damp,
                                                           float* __restrict__ lambda)
{
    __shared__ double s_part[256];
    double acc = 0.0;
    for (long i = threadIdx.x; i < K; i += 256) {
        const float dgl = hess[i * K + i];
        acc += (dgl == 0.0f) ? 1.0 : (double)dgl;
    }
    s_part[threadIdx.x] = acc;
    __syncthreads();
    for (int o = 128; o > 0; o >>= 1) {
        if ((int)threadIdx.x < o) s_part[threadIdx.x] += s_part[threadIdx.x + o];
        __syncthreads();
    }
    if (threadIdx.x == 0) *lambda = (float)((double)damp * s_part[0] / (double)K);
}

// v = J (H + damping) J
__global__ __launch_bounds__(256) void gptq_reverse_kernel(const float* __restrict__ hess, long K,
                                                           const float* __restrict__ lambda, float* __restrict__ v)
{
    const long at = (long)blockIdx.x * 256 + threadIdx.x;
    if (at >= K * K) return;
    const long i = at / K, j = at - i * K;
    float val = hess[(K - 1 - i) * K + (K - 1 - j)];
    if (i == j) val = ((val == 0.0f) ? 1.0f : val) + *lambda;
    v[at] = val;
}

__global__ __launch_bounds__(256) void gptq_fill_kernel(float* __restrict__ m, long K, float diag)
{
    const long at = (long)blockIdx.x * 256 + threadIdx.x;
    if (at >= K * K) return;
    const long i = at / K, j = at - i * K;
    m[at] = (i == j) ? diag : 0.0f;
}

// R_JJ^T R_JJ = A, A = the 64 x 64 diagonal block at (j0, j0) of v (its lower triangle is current), R_JJ
// written to r[(j0 + c) * K + j0 + j] (zeros below the diagonal).  One wavefront, lane j holds column j.
__global__ __launch_bounds__(kWave) void gptq_chol_diag_kernel(const float* __restrict__ v, long K, long j0,
                                                               float* __restrict__ r)
{
    const int j = threadIdx.x;
    float col[kGqGroup];                                          // A[i, j], read from the lower triangle
#pragma unroll
    for (int i = 0; i < kGqGroup; i++) col[i] = v[(j0 + max(i, j)) * K + j0 + min(i, j)];
    // row c of R is handed from lane to lane through LDS (one write, broadcast reads)
    __shared__ __attribute__((aligned(16))) float s_row[2][kGqGroup];
#pragma unroll
    for (int c = 0; c < kGqGroup; c++) {
        const float dcc = __shfl(col[c], c, kWave);
        const float rd = sqrtf(dcc);
        const float rj = (j >= c) ? col[c] / rd : 0.0f;           // R[c, j]
        r[(j0 + c) * K + j0 + j] = rj;
        s_row[c & 1][j] = rj;
        __syncthreads();                                          // one wavefront: orders the LDS write before the reads
#pragma unroll
        for (int i = c + 1; i < kGqGroup; i++) col[i] = __builtin_fmaf(-s_row[c & 1][i], rj, col[i]);
    }
}

}  // namespace dymoe

extern "C" {

size_t dymoe_gptq_workspace_bytes(long N, long K)
{
    if (N <= 0 || K <= 0) return 0;
    return dymoe::gq_round256((size_t)N * (size_t)K * 4) +
           dymoe::gq_round256(2 * (size_t)dymoe::kGqGroup * (size_t)dymoe::gq_rows_padded(N) * 4);
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
    const long G = K / kGqGroup;
    // one group of 64 columns: codes, scale, zero; its 64 errors per row go to err rows [64 * slot, 64 * slot + 64)
    auto group_step = [&](long base, int slot) {
        const float* xg = v + base;
        const float* dg = u + base * K + base;
        uint8_t* cg = codes + base * bits / 8;
        uint16_t* sg = (uint16_t*)scale + base / kGqGroup;
        uint16_t* zg = (uint16_t*)zero + base / kGqGroup;
        float* eg = err + (long)slot * kGqGroup * n_pad;
        float* const none = nullptr;
        switch (bits) {
        case 8:
            dymoe_launch(ctx, DYMOE_K_GPTQ_GROUP, (gptq_group_kernel<8, false, true>), grid_a, dim3(kGqRows), 0, st, xg, K, dg, K,
                         0L, N, none, 0L, 0L, eg, n_pad, 1L, cg, sg, zg, K * bits / 8, G);
            break;
        case 4:
            dymoe_launch(ctx, DYMOE_K_GPTQ_GROUP, (gptq_group_kernel<4, false, true>), grid_a, dim3(kGqRows), 0, st, xg, K, dg, K,
                         0L, N, none, 0L, 0L, eg, n_pad, 1L, cg, sg, zg, K * bits / 8, G);
            break;
        default:
            dymoe_launch(ctx, DYMOE_K_GPTQ_GROUP, (gptq_group_kernel<2, false, true>), grid_a, dim3(kGqRows), 0, st, xg, K, dg, K,
                         0L, N, none, 0L, 0L, eg, n_pad, 1L, cg, sg, zg, K * bits / 8, G);
            break;
        }
    };
    // corrections of `chunks` groups starting at column `base`, applied to the columns [col_begin, col_end)
    auto trail_step = [&](long base, int chunks, long col_begin, long col_end) {
        const dim3 grid_b((unsigned)((col_end - col_begin + kGqTrailCols - 1) / kGqTrailCols), (unsigned)(n_pad / kGqRows));
        dymoe_launch(ctx, DYMOE_K_GPTQ_TRAIL, gptq_trail_kernel, grid_b, dim3(kGqTrailThreads), 0, st, v, K,
                     (const float*)err, n_pad, u + base * K, K, 0L, N, col_begin, col_end, chunks, 0);
    };
    // Two groups per pass over the working copy: the first group's corrections reach the second group's 64 columns
    // at once, the second group is quantised, and both groups' 128 corrections then go over the remaining columns
    // together, in the same order as one group at a time (so the same roundings) at half the traffic.
    for (long base = 0; base < K; base += 2 * kGqGroup) {
        group_step(base, 0);
        DYMOE_HIP_LAUNCH_CHECK();
        if (base + kGqGroup >= K) break;
        trail_step(base, 1, base + kGqGroup, base + 2 * kGqGroup);
        group_step(base + kGqGroup, 1);
        DYMOE_HIP_LAUNCH_CHECK();
        if (base + 2 * kGqGroup < K) trail_step(base, 2, base + 2 * kGqGroup, K);
        DYMOE_HIP_LAUNCH_CHECK();
    }
    return DYMOE_OK;
}

int dymoe_gptq_hessian(dymoe_ctx* ctx, const void* x_bf16, long n, long K, int accumulate, float* hess, void* stream)
{
    using namespace dymoe;
    DYMOE_REQUIRE(x_bf16 && hess && n > 0 && K > 0 && K % 8 == 0 && (accumulate == 0 || accumulate == 1));
    DYMOE_REQUIRE(K <= 65536 && dymoe_aligned(x_bf16, 16) && dymoe_aligned(hess, 16));
    if (!ctx) return DYMOE_ENOCTX;
    const long nt = (K + kHsTile - 1) / kHsTile;
    dymoe_launch(ctx, DYMOE_K_GPTQ_HESSIAN, gptq_hessian_kernel, dim3((unsigned)(nt * (nt + 1) / 2)), dim3(kHsThreads), 0,
                 (hipStream_t)stream, (const uint16_t*)x_bf16, n, K, accumulate, hess);
    DYMOE_HIP_LAUNCH_CHECK();
    return DYMOE_OK;
}

size_t dymoe_gptq_factor_workspace_bytes(long K)
{
    if (K <= 0) return 0;
    // the reversed damped Hessian (later the substitution's right-hand sides), its Cholesky factor, 128 errors per row, damping
    return 2 * dymoe::gq_round256((size_t)K * (size_t)K * 4) + dymoe::gq_round256(2 * (size_t)dymoe::kGqGroup * (size_t)K * 4) + 256;
}

int dymoe_gptq_factor(dymoe_ctx* ctx, const float* hess, long K, float damp, float* u, void* workspace,
                      size_t workspace_bytes, void* stream)
{
    using namespace dymoe;
    DYMOE_REQUIRE(hess && u && workspace && K > 0 && K % kGqGroup == 0 && K <= 65536 && damp >= 0.0f);
    DYMOE_REQUIRE(dymoe_aligned(hess, 16) && dymoe_aligned(u, 16) && dymoe_aligned(workspace, 256));
    DYMOE_REQUIRE((const void*)hess != (const void*)u);
    if (workspace_bytes < dymoe_gptq_factor_workspace_bytes(K)) return DYMOE_ENOSPC;
    if (!ctx) return DYMOE_ENOCTX;
    hipStream_t st = (hipStream_t)stream;
    const size_t mat = gq_round256((size_t)K * (size_t)K * 4);
    float* v = reinterpret_cast<float*>(workspace);
    float* r = reinterpret_cast<float*>((char*)workspace + mat);
    float* err = reinterpret_cast<float*>((char*)workspace + 2 * mat);
    float* lambda = reinterpret_cast<float*>((char*)workspace + 2 * mat + gq_round256(2 * (size_t)kGqGroup * (size_t)K * 4));
    const dim3 whole((unsigned)((K * K + 255) / 256));
    hipLaunchKernelGGL(gptq_damping_kernel, dim3(1), dim3(256), 0, st, hess, K, damp, lambda);
    hipLaunchKernelGGL(gptq_reverse_kernel, whole, dim3(256), 0, st, hess, K, (const float*)lambda, v);
    hipLaunchKernelGGL(gptq_fill_kernel, whole, dim3(256), 0, st, r, K, 0.0f);
    DYMOE_HIP_LAUNCH_CHECK();
    float* const none = nullptr;
    // (both loops take two blocks of 64 per pass over the trailing matrix, as the quantizer's sweep does)
    auto trail = [&](long row_begin, long row_end, long col_begin, long col_end, const float* e, long lde, const float* b,
                     int chunks, int lower_only) {
        const dim3 grid_b((unsigned)((col_end - col_begin + kGqTrailCols - 1) / kGqTrailCols),
                          (unsigned)((row_end - row_begin) / kGqRows));
        dymoe_launch(ctx, DYMOE_K_GPTQ_TRAIL, gptq_trail_kernel, grid_b, dim3(kGqTrailThreads), 0, st, v, K, e, lde, b, K,
                     row_begin, row_end, col_begin, col_end, chunks, lower_only);
    };
    // J (H + damping) J = R^T R
    // diagonal block at j0, then the rows below it solved against it: the panel of L goes into R as rows,
    // L[row, j0 + c] = R[j0 + c, row]
    auto chol_block = [&](long j0) {
        dymoe_launch(ctx, DYMOE_K_GPTQ_FACTOR, gptq_chol_diag_kernel, dim3(1), dim3(kWave), 0, st, (const float*)v, K, j0, r);
        const long below = K - j0 - kGqGroup;
        if (below > 0)
            dymoe_launch(ctx, DYMOE_K_GPTQ_GROUP, (gptq_group_kernel<0, true, false>), dim3((unsigned)(below / kGqRows)),
                         dim3(kGqRows), 0, st, (const float*)(v + j0), K, (const float*)(r + j0 * K + j0), K, j0 + kGqGroup, K,
                         r + j0 * K, K, 1L, none, 0L, 0L, (uint8_t*)nullptr, (uint16_t*)nullptr, (uint16_t*)nullptr, 0L, 0L);
    };
    for (long j0 = 0; j0 < K; j0 += 2 * kGqGroup) {
        const long j1 = j0 + kGqGroup, j2 = j0 + 2 * kGqGroup;
        chol_block(j0);
        DYMOE_HIP_LAUNCH_CHECK();
        if (j1 >= K) break;
        trail(j1, K, j1, j2, r + j0 * K, K, r + j0 * K, 1, 1);          // the next block's columns first
        chol_block(j1);
        DYMOE_HIP_LAUNCH_CHECK();
        if (j2 < K) trail(j2, K, j2, K, r + j0 * K, K, r + j0 * K, 2, 1);  // then both panels over the rest of the lower triangle
        DYMOE_HIP_LAUNCH_CHECK();
    }
    // rows of R^-T by forward substitution of the unit vectors, mirrored into U
    hipLaunchKernelGGL(gptq_fill_kernel, whole, dim3(256), 0, st, v, K, 1.0f);
    hipLaunchKernelGGL(gptq_fill_kernel, whole, dim3(256), 0, st, u, K, 0.0f);
    DYMOE_HIP_LAUNCH_CHECK();
    // one block of 64 columns for the rows [0, rows): e of (row c, column base + i) is U[K - 1 - base - i, K - 1 - c];
    // rows that have not started yet (c >= base + 64) hold zeros there and give e = 0
    auto subst_block = [&](long base, long rows, int slot) {
        dymoe_launch(ctx, DYMOE_K_GPTQ_GROUP, (gptq_group_kernel<0, true, true>), dim3((unsigned)(rows / kGqRows)), dim3(kGqRows),
                     0, st, (const float*)(v + base), K, (const float*)(r + base * K + base), K, 0L, rows,
                     u + (K - 1 - base) * K + (K - 1), -K, -1L, err + (long)slot * kGqGroup * K, K, 1L, (uint8_t*)nullptr,
                     (uint16_t*)nullptr, (uint16_t*)nullptr, 0L, 0L);
    };
    for (long base = 0; base < K; base += 2 * kGqGroup) {
        const long b1 = base + kGqGroup, b2 = base + 2 * kGqGroup;
        const long rows = (b2 < K) ? b2 : K;
        subst_block(base, rows, 0);
        DYMOE_HIP_LAUNCH_CHECK();
        if (b1 >= K) break;
        trail(0, b1, b1, b2, err, K, r + base * K, 1, 0);
        subst_block(b1, rows, 1);
        DYMOE_HIP_LAUNCH_CHECK();
        if (b2 < K) trail(0, b2, b2, K, err, K, r + base * K, 2, 0);
        DYMOE_HIP_LAUNCH_CHECK();
    }
    return DYMOE_OK;
}

}  // extern "C"
