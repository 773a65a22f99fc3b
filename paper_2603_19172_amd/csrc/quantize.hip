// Group-wise asymmetric quantize-and-pack (bf16 -> int4 / int2 codes + fp16
// scale and zero per group of 64 columns).  Streaming kernel: every lane owns
// 32 consecutive bf16 (four 16-byte loads, 64 contiguous bytes), two lanes own
// a group, and a lane writes its 32 codes with one 16-byte (int4) or 8-byte
// (int2) store.
//
// The arithmetic is an exact sequence of binary32 operations (this file is
// built with -ffp-contract=off): the codes must equal the reference's bit for
// bit, so nothing here may be fused, reassociated or approximated.
//   round-to-nearest-even of v = (w - m) * inv is done by the addition
//   v + 1.5*2^23, which is exact RNE-to-integer for |v| < 2^22 and leaves the
//   integer in the low mantissa bits; the clamp then runs on the bit pattern.
#include "common.hpp"

namespace dymoe {

constexpr int kQThreads = 256;
constexpr int kQElemsPerLane = 32;
constexpr int kQElemsPerBlock = kQThreads * kQElemsPerLane;  // 8192 elements = 128 groups
constexpr int kRowStageLane = 64;                            // bytes of a lane's 32 weights in the LDS stage
constexpr int kRowStageBytes = kWave * kRowStageLane;        // per wavefront

__device__ __forceinline__ void unpack8(const uint4 raw, float* v)
{
    v[0] = bf16_lo(raw.x); v[1] = bf16_hi(raw.x);
    v[2] = bf16_lo(raw.y); v[3] = bf16_hi(raw.y);
    v[4] = bf16_lo(raw.z); v[5] = bf16_hi(raw.z);
    v[6] = bf16_lo(raw.w); v[7] = bf16_hi(raw.w);
}

// One block quantizes elements [block*8192, block*8192 + 8192) of a matrix
// whose element count is a multiple of 64 (rows are whole groups, so the flat
// element index addresses the packed row-major outputs directly).
template <int BITS>
__device__ __forceinline__ void quantize_block(const uint16_t* __restrict__ w, long n_elems,
                                               uint8_t* __restrict__ codes,
                                               uint16_t* __restrict__ scale,
                                               uint16_t* __restrict__ zero, long block, uint8_t* stage)
{
#pragma clang fp contract(off)
    constexpr int qmax = (1 << BITS) - 1;
    constexpr float kMagic = 12582912.0f;          // 1.5 * 2^23
    constexpr int kMagicBits = 0x4B400000;
    const int lane = threadIdx.x & (kWave - 1);
    const long e0 = block * (long)kQElemsPerBlock + (long)threadIdx.x * kQElemsPerLane;
    // The wavefront's 4 KiB come in with whole-line loads (lane l takes 16 bytes of each of four 1 KiB pieces) and
    // are turned through the wavefront's LDS stage into 32 consecutive weights per lane.  Within a lane's 64 bytes
    // the four 16-byte pieces are stored in the order piece ^ ((lane >> 2) & 3): lanes 4 apart, whose 64 bytes
    // start in the same banks, then read different quarters, and neither the writes nor the reads conflict.
    uint4 raw[4];
    {
        const long wave0 = e0 - (long)lane * kQElemsPerLane;      // first element of the wavefront
#pragma unroll
        for (int c = 0; c < 4; c++) {
            const long at = wave0 + (long)(c * kWave + lane) * 8;
            raw[c] = make_uint4(0, 0, 0, 0);
            if (at < n_elems) raw[c] = load_global_nt<uint4>(w + at);
        }
#pragma unroll
        for (int c = 0; c < 4; c++)
            *reinterpret_cast<uint4*>(stage + (16 * c + (lane >> 2)) * kRowStageLane +
                                      (((lane & 3) ^ ((lane >> 4) & 3)) * 16)) = raw[c];   // owner lane 16 c + lane / 4
        __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "wavefront");      // the stage is the wavefront's own
        __builtin_amdgcn_wave_barrier();
#pragma unroll
        for (int c = 0; c < 4; c++)
            raw[c] = *reinterpret_cast<const uint4*>(stage + lane * kRowStageLane + ((c ^ ((lane >> 2) & 3)) * 16));
        __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "wavefront");      // read before the next block overwrites it
        __builtin_amdgcn_wave_barrier();
    }
    // a group's two lanes are in or out together (n_elems is a multiple of 64)
    if (e0 >= n_elems) return;
    float v[32];
#pragma unroll
    for (int c = 0; c < 4; c++) unpack8(raw[c], v + 8 * c);
    float lo = v[0], hi = v[0];
#pragma unroll
    for (int i = 1; i < 32; i++) {
        lo = fminf(lo, v[i]);
        hi = fmaxf(hi, v[i]);
    }
    lo = fminf(lo, __shfl_xor(lo, 1, kWave));
    hi = fmaxf(hi, __shfl_xor(hi, 1, kWave));
    const _Float16 zh = (_Float16)lo;                 // round to nearest even
    const float range = hi - lo;
    const float step = range / (float)qmax;           // correctly rounded division
    const _Float16 sh = (_Float16)step;
    const float m = (float)zh;
    const float s = (float)sh;
    const float inv = (s > 0.0f) ? (1.0f / s) : 0.0f;
    uint32_t words[BITS];                             // 32 codes: 8 words (int8), 4 (int4) or 2 (int2)
#pragma unroll
    for (int wd = 0; wd < BITS; wd++) {
        constexpr int per_word = 32 / BITS;
        uint32_t bytes[4];
#pragma unroll
        for (int b = 0; b < 4; b++) {
            constexpr int per_byte = 8 / BITS;
            uint32_t acc = 0;
#pragma unroll
            for (int j = per_byte - 1; j >= 0; j--) {
                const int i = wd * per_word + b * per_byte + j;
                const float d = v[i] - m;
                const float t = d * inv;
                const float r = t + kMagic;
                int q = __float_as_int(r);
                q = min(max(q, kMagicBits), kMagicBits + qmax);
                // the low byte accumulates the codes; bits above it are garbage
                acc = (j == per_byte - 1) ? (uint32_t)q : ((acc << BITS) | (uint32_t)q);
            }
            bytes[b] = acc;
        }
        // gather the four low bytes
        const uint32_t lo16 = __builtin_amdgcn_perm(bytes[1], bytes[0], 0x0c0c0400u);
        const uint32_t hi16 = __builtin_amdgcn_perm(bytes[3], bytes[2], 0x04000c0cu);
        words[wd] = lo16 | hi16;
    }
    if constexpr (BITS == 8) {
        store_global_nt(codes + e0, make_uint4(words[0], words[1], words[2], words[3]));
        store_global_nt(codes + e0 + 16, make_uint4(words[4], words[5], words[6], words[7]));
    } else if constexpr (BITS == 4) {
        store_global_nt(codes + (e0 >> 1), make_uint4(words[0], words[1], words[2], words[3]));
    } else {
        store_global_nt(codes + (e0 >> 2), make_uint2(words[0], words[1]));
    }
    // The wavefront's 32 scales and 32 zeros leave as 16-byte non-temporal stores: lane 16 i gathers the scales of
    // the eight groups held by lanes 16 i .. 16 i + 15, lane 16 i + 1 their zeros (a wavefront whose tail lies past
    // the end of the matrix has returned above as a whole or holds only whole groups of eight: n_elems is a
    // multiple of 64, and a wavefront covers 32 groups, so a partial one is handled by the plain stores below).
    const uint32_t mine = (lane & 1) ? 0u : ((uint32_t)(uint16_t)f16_bits(sh) | ((uint32_t)(uint16_t)f16_bits(zh) << 16));
    const long wave_e0 = e0 - (long)lane * kQElemsPerLane;
    if (wave_e0 + (long)kWave * kQElemsPerLane <= n_elems && (((uintptr_t)scale | (uintptr_t)zero) & 15) == 0) {
        const int base = lane & ~15;
        uint32_t g[8];
#pragma unroll
        for (int i = 0; i < 8; i++) g[i] = (uint32_t)__shfl((int)mine, base + 2 * i, kWave);
        const int which = lane & 15;                 // 0: scales, 1: zeros of this run of eight groups
        if (which < 2) {
            uint32_t h[8];
#pragma unroll
            for (int i = 0; i < 8; i++) h[i] = which ? (g[i] >> 16) : (g[i] & 0xffffu);
            const uint4 out = make_uint4(h[0] | (h[1] << 16), h[2] | (h[3] << 16), h[4] | (h[5] << 16), h[6] | (h[7] << 16));
            uint16_t* dst = (which ? zero : scale) + (wave_e0 >> 6) + (lane >> 4) * 8;
            store_global_nt(dst, out);
        }
    } else if ((lane & 1) == 0) {
        store_global(scale + (e0 >> 6), (uint16_t)f16_bits(sh));
        store_global(zero + (e0 >> 6), (uint16_t)f16_bits(zh));
    }
}

__global__ __launch_bounds__(kQThreads) void quantize_pack_kernel(
    const uint16_t* __restrict__ w, long n_elems, int bits,
    uint8_t* __restrict__ codes, uint16_t* __restrict__ scale, uint16_t* __restrict__ zero)
{
    __shared__ __attribute__((aligned(16))) uint8_t stage[(kQThreads / kWave) * kRowStageBytes];
    uint8_t* mine = stage + (threadIdx.x / kWave) * kRowStageBytes;
    if (bits == 8) quantize_block<8>(w, n_elems, codes, scale, zero, blockIdx.x, mine);
    else if (bits == 4) quantize_block<4>(w, n_elems, codes, scale, zero, blockIdx.x, mine);
    else quantize_block<2>(w, n_elems, codes, scale, zero, blockIdx.x, mine);
}

// Tile-layout variant: a lane owns a whole group (row 32*nt + r, columns
// 128*kt + 64*kb .. +64 of tile (nt, kt), lane l = 32*kb + r), no cross-lane
// arithmetic, and the codes, scale and zero go to the lane's slots of the tile.
// One wavefront per tile.  The tile's 32 row pieces of 256 bytes are fetched
// with whole-line loads (16 lanes per row piece, 4 rows per instruction) and
// turned through the wavefront's LDS stage into the lane-owns-a-group order;
// rows of the stage are 272 bytes apart so that neither side has bank conflicts.
constexpr int kTileStageRow = 272;
constexpr int kTileStageBytes = 32 * kTileStageRow;

template <int BITS>
__device__ __forceinline__ void quantize_tile(const uint16_t* __restrict__ w, long K, long tile,
                                              uint8_t* __restrict__ codes,
                                              uint16_t* __restrict__ scale,
                                              uint16_t* __restrict__ zero, uint8_t* stage)
{
#pragma clang fp contract(off)
    constexpr int qmax = (1 << BITS) - 1;
    constexpr float kMagic = 12582912.0f;          // 1.5 * 2^23
    constexpr int kMagicBits = 0x4B400000;
    const int lane = threadIdx.x & (kWave - 1);
    const long KT = K >> 7;
    const long nt = tile / KT;
    const long kt = tile - nt * KT;
    uint4 raw[8];
    {
        const uint16_t* src = w + (nt * 32 + (lane >> 4)) * K + kt * 128 + (lane & 15) * 8;
#pragma unroll
        for (int c = 0; c < 8; c++) raw[c] = load_global_nt<uint4>(src + 4 * c * K);
        uint8_t* put = stage + (lane >> 4) * kTileStageRow + (lane & 15) * 16;
#pragma unroll
        for (int c = 0; c < 8; c++) *reinterpret_cast<uint4*>(put + 4 * c * kTileStageRow) = raw[c];
        __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "wavefront");      // the stage is the wavefront's own
        __builtin_amdgcn_wave_barrier();
        const uint8_t* get = stage + (lane & 31) * kTileStageRow + (lane >> 5) * 128;
#pragma unroll
        for (int c = 0; c < 8; c++) raw[c] = *reinterpret_cast<const uint4*>(get + 16 * c);
        __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "wavefront");      // read before the next tile overwrites it
        __builtin_amdgcn_wave_barrier();
    }
    float v[64];
#pragma unroll
    for (int c = 0; c < 8; c++) unpack8(raw[c], v + 8 * c);
    float lo = v[0], hi = v[0];
#pragma unroll
    for (int i = 1; i < 64; i++) {
        lo = fminf(lo, v[i]);
        hi = fmaxf(hi, v[i]);
    }
    const _Float16 zh = (_Float16)lo;                 // round to nearest even
    const float range = hi - lo;
    const float step = range / (float)qmax;           // correctly rounded division
    const _Float16 sh = (_Float16)step;
    const float m = (float)zh;
    const float s = (float)sh;
    const float inv = (s > 0.0f) ? (1.0f / s) : 0.0f;
    constexpr int kWords = 2 * BITS;                  // 64 codes: 16 words (int8), 8 (int4) or 4 (int2)
    uint32_t words[kWords];
#pragma unroll
    for (int wd = 0; wd < kWords; wd++) {
        constexpr int per_word = 32 / BITS;
        uint32_t bytes[4];
#pragma unroll
        for (int b = 0; b < 4; b++) {
            constexpr int per_byte = 8 / BITS;
            uint32_t acc = 0;
#pragma unroll
            for (int j = per_byte - 1; j >= 0; j--) {
                const int i = wd * per_word + b * per_byte + j;
                const float d = v[i] - m;
                const float t = d * inv;
                const float r = t + kMagic;
                int q = __float_as_int(r);
                q = min(max(q, kMagicBits), kMagicBits + qmax);
                acc = (j == per_byte - 1) ? (uint32_t)q : ((acc << BITS) | (uint32_t)q);
            }
            bytes[b] = acc;
        }
        const uint32_t lo16 = __builtin_amdgcn_perm(bytes[1], bytes[0], 0x0c0c0400u);
        const uint32_t hi16 = __builtin_amdgcn_perm(bytes[3], bytes[2], 0x04000c0cu);
        words[wd] = lo16 | hi16;
    }
    if constexpr (BITS == 8) {
        uint8_t* dst = codes + tile * 4096 + lane * 16;
#pragma unroll
        for (int c = 0; c < 4; c++)
            store_global_nt(dst + c * 1024, make_uint4(words[4 * c], words[4 * c + 1], words[4 * c + 2], words[4 * c + 3]));
    } else if constexpr (BITS == 4) {
        uint8_t* dst = codes + tile * 2048 + lane * 16;
        store_global_nt(dst, make_uint4(words[0], words[1], words[2], words[3]));
        store_global_nt(dst + 1024, make_uint4(words[4], words[5], words[6], words[7]));
    } else {
        store_global_nt(codes + tile * 1024 + lane * 16, make_uint4(words[0], words[1], words[2], words[3]));
    }
    // the tile's 64 scales and 64 zeros (128 bytes each) leave as 16-byte non-temporal stores: lane 8 i gathers the
    // scales of lanes 8 i .. 8 i + 7, lane 8 i + 1 their zeros
    if ((((uintptr_t)scale | (uintptr_t)zero) & 15) == 0) {
        const uint32_t mine = (uint32_t)(uint16_t)f16_bits(sh) | ((uint32_t)(uint16_t)f16_bits(zh) << 16);
        const int base = lane & ~7;
        uint32_t g[8];
#pragma unroll
        for (int i = 0; i < 8; i++) g[i] = (uint32_t)__shfl((int)mine, base + i, kWave);
        const int which = lane & 7;                  // 0: scales, 1: zeros of this run of eight groups
        if (which < 2) {
            uint32_t h[8];
#pragma unroll
            for (int i = 0; i < 8; i++) h[i] = which ? (g[i] >> 16) : (g[i] & 0xffffu);
            const uint4 out = make_uint4(h[0] | (h[1] << 16), h[2] | (h[3] << 16), h[4] | (h[5] << 16), h[6] | (h[7] << 16));
            store_global_nt((which ? zero : scale) + tile * 64 + base, out);
        }
    } else {
        store_global(scale + tile * 64 + lane, (uint16_t)f16_bits(sh));
        store_global(zero + tile * 64 + lane, (uint16_t)f16_bits(zh));
    }
}

// bf16 row-major -> bf16 tiles: thread = (tile, chunk j, lane)
__global__ __launch_bounds__(256) void pack_tiles_kernel(const uint16_t* __restrict__ w, long N,
                                                         long K, uint16_t* __restrict__ tiles)
{
    const long i = (long)blockIdx.x * 256 + threadIdx.x;     // one 16-byte chunk of the output
    if (i >= N * K / 8) return;
    const long tile = i >> 9;                                  // 512 chunks per tile
    const int j = (int)((i >> 6) & 7);
    const int lane = (int)(i & 63);
    const long KT = K >> 7;
    const long nt = tile / KT;
    const long kt = tile - nt * KT;
    const long row = nt * 32 + (lane & 31);
    const long col = kt * 128 + 64 * (lane >> 5) + 8 * j;
    reinterpret_cast<uint4*>(tiles)[i] = *reinterpret_cast<const uint4*>(w + row * K + col);
}

// packed codes + scale + zero, row-major -> tile layout: thread = (tile, lane); a lane's group is contiguous in
// both layouts (8 * bits bytes), so the move is bits / 2 16-byte copies and two 2-byte ones
__global__ __launch_bounds__(256) void pack_code_tiles_kernel(
    const uint8_t* __restrict__ codes, const uint16_t* __restrict__ scale, const uint16_t* __restrict__ zero, long N,
    long K, int bits, uint8_t* __restrict__ t_codes, uint16_t* __restrict__ t_scale, uint16_t* __restrict__ t_zero)
{
    const long i = (long)blockIdx.x * 256 + threadIdx.x;
    if (i >= N * K / 64) return;                              // one group per thread
    const long tile = i >> 6;
    const int lane = (int)(i & 63);
    const long KT = K >> 7;
    const long nt = tile / KT;
    const long kt = tile - nt * KT;
    const long row = nt * 32 + (lane & 31);
    const long grp = kt * 2 + (lane >> 5);
    const uint8_t* src = codes + row * (K * bits / 8) + grp * (8 * bits);
    uint8_t* dst = t_codes + tile * (512 * bits) + lane * 16;
    for (int c = 0; c < bits / 2; c++) store_global(dst + c * 1024, load_global<uint4>(src + 16 * c));
    t_scale[tile * 64 + lane] = scale[row * (K >> 6) + grp];
    t_zero[tile * 64 + lane] = zero[row * (K >> 6) + grp];
}

// Worklist of a layer: the experts whose assigned width is 8, 4 or 2 bits (and
// that have load, when load is given), in ascending order.  Every workgroup
// builds its own copy in LDS with its first wavefront (ballot + prefix count),
// so no separate launch and no global buffer is needed.  Returns the count.
__device__ __forceinline__ int build_worklist(const uint8_t* __restrict__ bits,
                                              const int32_t* __restrict__ load, int E,
                                              int16_t* list, int* count)
{
    if (threadIdx.x < kWave) {
        const int lane = threadIdx.x;
        int n = 0;
        for (int base = 0; base < E; base += kWave) {
            const int e = base + lane;
            bool need = false;
            if (e < E) {
                const int b = bits[e];
                need = (b == 8 || b == 4 || b == 2) && (load == nullptr || load[e] > 0);
            }
            const unsigned long long mask = __ballot(need);
            if (need) list[n + __popcll(mask & ((1ull << lane) - 1ull))] = (int16_t)e;
            n += __popcll(mask);
        }
        if (lane == 0) *count = n;
    }
    __syncthreads();
    return *count;
}

// A fixed-size grid walks (expert of the worklist, matrix, block) units, so no
// workgroup is launched for experts that need nothing and the precision
// decision never goes through the host.
template <int LAYOUT>
__global__ __launch_bounds__(kQThreads) void quantize_experts_kernel(
    const dymoe_expert_fmt* __restrict__ table, const uint8_t* __restrict__ bits,
    const int32_t* __restrict__ load, int E, int H, int F, unsigned* __restrict__ flags)
{
    __shared__ int16_t list[DYMOE_MAX_EXPERTS];
    __shared__ int n_list;
    __shared__ __attribute__((aligned(16))) uint8_t
        stage[(kQThreads / kWave) * ((LAYOUT == DYMOE_LAYOUT_TILE) ? kTileStageBytes : kRowStageBytes)];
    const int n_work = build_worklist(bits, load, E, list, &n_list);
    const long n_elems = (long)H * (long)F;
    // row-major: 8192 elements per block; tiles: 4 tiles (one per wavefront) = 16384 elements
    constexpr long kPerBlock = (LAYOUT == DYMOE_LAYOUT_TILE) ? 4 * 4096 : kQElemsPerBlock;
    const long bpm = (n_elems + kPerBlock - 1) / kPerBlock;               // blocks per matrix
    const long units = (long)n_work * 3 * bpm;
    for (long u = blockIdx.x; u < units; u += gridDim.x) {
        const long item = u / bpm;
        const long blk = u - item * bpm;
        const int e = list[item / 3];
        const int mat = (int)(item % 3);
        const int b = bits[e];
        const dymoe_expert_fmt* ex = table + e;
        const uint16_t* w = reinterpret_cast<const uint16_t*>(ex->w[mat]);
        uint8_t* q = (b == 8) ? ex->q8[mat] : (b == 4) ? ex->q4[mat] : ex->q2[mat];
        uint16_t* sc = reinterpret_cast<uint16_t*>((b == 8) ? ex->s8[mat] : (b == 4) ? ex->s4[mat] : ex->s2[mat]);
        uint16_t* zr = reinterpret_cast<uint16_t*>((b == 8) ? ex->z8[mat] : (b == 4) ? ex->z4[mat] : ex->z2[mat]);
        if (!w || !q || !sc || !zr) {         // no source, or nowhere to write the selected format: nothing is written
            if (blk == 0 && threadIdx.x == 0) atomicOr(flags, DYMOE_FLAG_FORMAT_MISSING);
            continue;                          // (the same for every thread of the workgroup)
        }
        if constexpr (LAYOUT == DYMOE_LAYOUT_TILE) {
            const long K = (mat == 2) ? F : H;
            const long tile = blk * 4 + (threadIdx.x >> 6);
            if (tile * 4096 < n_elems) {
                uint8_t* mine = stage + (threadIdx.x >> 6) * kTileStageBytes;
                if (b == 8) quantize_tile<8>(w, K, tile, q, sc, zr, mine);
                else if (b == 4) quantize_tile<4>(w, K, tile, q, sc, zr, mine);
                else quantize_tile<2>(w, K, tile, q, sc, zr, mine);
            }
        } else {
            uint8_t* mine = stage + (threadIdx.x >> 6) * kRowStageBytes;
            if (b == 8) quantize_block<8>(w, n_elems, q, sc, zr, blk, mine);
            else if (b == 4) quantize_block<4>(w, n_elems, q, sc, zr, blk, mine);
            else quantize_block<2>(w, n_elems, q, sc, zr, blk, mine);
        }
    }
}

}  // namespace dymoe

extern "C" {

int dymoe_quantize_pack(dymoe_ctx* ctx, const void* w, long N, long K, int bits, int group,
                        uint8_t* codes, void* scale, void* zero, void* stream)
{
    DYMOE_REQUIRE(N >= 0 && K > 0);
    DYMOE_REQUIRE(bits == 2 || bits == 4 || bits == 8);
    DYMOE_REQUIRE(group > 0 && K % group == 0);
    if (N == 0) return (group != 64) ? DYMOE_ENOTSUP : (ctx ? DYMOE_OK : DYMOE_ENOCTX);  // nothing to read or write
    DYMOE_REQUIRE(w && codes && scale && zero);
    DYMOE_REQUIRE(dymoe_aligned(w, 16) && dymoe_aligned(codes, 16) && dymoe_aligned(scale, 2) &&
                  dymoe_aligned(zero, 2));
    if (group != 64) return DYMOE_ENOTSUP;
    if (!ctx) return DYMOE_ENOCTX;
    const long n_elems = N * K;
    const long blocks = (n_elems + dymoe::kQElemsPerBlock - 1) / dymoe::kQElemsPerBlock;
    if (blocks > 0x7fffffffL) return DYMOE_ENOTSUP;
    dymoe_launch(ctx, DYMOE_K_QUANTIZE, dymoe::quantize_pack_kernel, dim3((unsigned)blocks), dim3(dymoe::kQThreads), 0,
                       (hipStream_t)stream, (const uint16_t*)w, n_elems, bits, codes,
                       (uint16_t*)scale, (uint16_t*)zero);
    DYMOE_HIP_LAUNCH_CHECK();
    return DYMOE_OK;
}

int dymoe_quantize_experts(dymoe_ctx* ctx, const dymoe_expert_fmt* table, const uint8_t* bits,
                           const int32_t* load, int E, int H, int F, int group, int layout,
                           void* stream)
{
    DYMOE_REQUIRE(table && bits);
    DYMOE_REQUIRE(E > 0 && H > 0 && F > 0);
    DYMOE_REQUIRE(group > 0 && H % group == 0 && F % group == 0);
    DYMOE_REQUIRE(layout == DYMOE_LAYOUT_ROWMAJOR || layout == DYMOE_LAYOUT_TILE);
    if (layout == DYMOE_LAYOUT_TILE) DYMOE_REQUIRE(H % 128 == 0 && F % 128 == 0);
    if (group != 64 || E > DYMOE_MAX_EXPERTS) return DYMOE_ENOTSUP;
    if (!ctx) return DYMOE_ENOCTX;
    hipStream_t st = (hipStream_t)stream;
    const long n_elems = (long)H * (long)F;
    const long per_block = (layout == DYMOE_LAYOUT_TILE) ? 4 * 4096 : dymoe::kQElemsPerBlock;
    const long bpm = (n_elems + per_block - 1) / per_block;
    long grid = 3L * E * bpm;
    const long cap = (long)ctx->num_cu * 32;   // enough resident workgroups to fill the chip; the rest loops
    if (grid > cap) grid = cap;
    if (layout == DYMOE_LAYOUT_TILE)
        dymoe_launch(ctx, DYMOE_K_QUANTIZE, dymoe::quantize_experts_kernel<DYMOE_LAYOUT_TILE>,
                     dim3((unsigned)grid), dim3(dymoe::kQThreads), 0, st, table, bits, load, E, H, F, ctx->device_flags);
    else
        dymoe_launch(ctx, DYMOE_K_QUANTIZE, dymoe::quantize_experts_kernel<DYMOE_LAYOUT_ROWMAJOR>,
                     dim3((unsigned)grid), dim3(dymoe::kQThreads), 0, st, table, bits, load, E, H, F, ctx->device_flags);
    DYMOE_HIP_LAUNCH_CHECK();
    return DYMOE_OK;
}

int dymoe_pack_tiles(dymoe_ctx* ctx, const void* w, long N, long K, void* tiles, void* stream)
{
    DYMOE_REQUIRE(N >= 0 && K > 0 && N % 32 == 0 && K % 128 == 0);
    if (N == 0) return ctx ? DYMOE_OK : DYMOE_ENOCTX;
    DYMOE_REQUIRE(w && tiles && w != tiles);
    DYMOE_REQUIRE(dymoe_aligned(w, 16) && dymoe_aligned(tiles, 16));
    if (!ctx) return DYMOE_ENOCTX;
    const long chunks = N * K / 8;
    const long blocks = (chunks + 255) / 256;
    if (blocks > 0x7fffffffL) return DYMOE_ENOTSUP;
    hipLaunchKernelGGL(dymoe::pack_tiles_kernel, dim3((unsigned)blocks), dim3(256), 0,
                       (hipStream_t)stream, (const uint16_t*)w, N, K, (uint16_t*)tiles);
    DYMOE_HIP_LAUNCH_CHECK();
    return DYMOE_OK;
}

int dymoe_pack_code_tiles(dymoe_ctx* ctx, const uint8_t* codes, const void* scale, const void* zero, long N, long K,
                          int bits, uint8_t* t_codes, void* t_scale, void* t_zero, void* stream)
{
    DYMOE_REQUIRE(N >= 0 && K > 0 && N % 32 == 0 && K % 128 == 0 && (bits == 2 || bits == 4 || bits == 8));
    if (N == 0) return ctx ? DYMOE_OK : DYMOE_ENOCTX;
    DYMOE_REQUIRE(codes && scale && zero && t_codes && t_scale && t_zero);
    DYMOE_REQUIRE(codes != t_codes && scale != t_scale && zero != t_zero);
    DYMOE_REQUIRE(dymoe_aligned(codes, 16) && dymoe_aligned(t_codes, 16) && dymoe_aligned(scale, 2) &&
                  dymoe_aligned(zero, 2) && dymoe_aligned(t_scale, 2) && dymoe_aligned(t_zero, 2));
    if (!ctx) return DYMOE_ENOCTX;
    const long blocks = (N * K / 64 + 255) / 256;
    if (blocks > 0x7fffffffL) return DYMOE_ENOTSUP;
    hipLaunchKernelGGL(dymoe::pack_code_tiles_kernel, dim3((unsigned)blocks), dim3(256), 0, (hipStream_t)stream, codes,
                       (const uint16_t*)scale, (const uint16_t*)zero, N, K, bits, t_codes, (uint16_t*)t_scale,
                       (uint16_t*)t_zero);
    DYMOE_HIP_LAUNCH_CHECK();
    return DYMOE_OK;
}

}  // extern "C"
