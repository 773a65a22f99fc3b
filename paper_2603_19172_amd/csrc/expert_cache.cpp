// Mixed-precision expert cache with one byte budget (paper Sec. 4.4.2).
// Host-side bookkeeping only: no GPU call, no device memory.  The caller owns an
// arena of `budget_bytes` of device memory and copies experts into the slots
// this cache hands out (as byte offsets into that arena).
//
// The three rules of the paper:
//   No Duplication       an expert is resident in at most one format;
//   Precision Promotion  a request above the resident precision is a miss: the
//                        higher format is loaded, the lower one dropped;
//   Conservative Reuse   a request at or below the resident precision is a hit
//                        and the resident (higher) format is used.
//
// One budget, several slot sizes: the arena is cut into blocks of the largest
// slot size; a block belongs to one format at a time and holds as many slots of
// that format as fit.  A request first takes a free slot of its format, then a
// free block; otherwise it evicts the least recently used of
//   (a) the unprotected residents of its own format, and
//   (b) the blocks of other formats none of whose residents is protected, a
//       block being as recent as its most recently used resident,
// (a) on equal age.  Evicting a block frees all its slots and hands the block
// over to the requesting format.
//
// Which resident goes first is least-recently-used order (the paper extends the standard LRU cache), or, when the
// caller says that requests walk a cyclic schedule of positions (dymoe_cache_set_cyclic: the layers of a decoder,
// visited 0, 1, ..., L-1, 0, ...), the resident whose position comes up last: a stack of layers touches every layer's
// experts once per step, and when a step's working set exceeds the cache, LRU order evicts each entry shortly before
// its layer comes round again and never hits, while "farthest next visit first" keeps the layers just ahead.
//
// The same rules over a FIXED partition (dymoe_cache_create_pools): so many
// slots per format, each slot a block of its own that never changes hands; room
// for a request then comes from its own format's pool alone.
#include "dymoe.h"

#include <stdint.h>

#include <algorithm>
#include <new>
#include <unordered_map>
#include <vector>

namespace {

struct Resident {
    int fmt;        // index into the format table
    int block;
    int slot;
    uint64_t tick;  // time of last use
    int pos;        // position of the cyclic schedule it was last asked for at (0 without a schedule)
};

struct Block {
    int fmt = -1;                 // -1: free
    int used = 0;
    int pin = -1;                 // fixed partition: the only format this block ever serves (-1: any)
    size_t base = 0;              // byte offset of the block in the arena
    std::vector<int64_t> keys;    // per slot: resident key, or kNoKey
};

constexpr int64_t kNoKey = INT64_MIN;

}  // namespace

struct dymoe_cache {
    std::vector<int> bits;             // per format, descending precision not required
    std::vector<size_t> slot_bytes;    // per format, rounded up to 256
    std::vector<int> slots_per_block;
    size_t block_bytes = 0;
    std::vector<Block> blocks;
    std::unordered_map<int64_t, Resident> where;
    uint64_t clock = 0;
    int n_pos = 0;                     // length of the cyclic schedule (0: none, least recently used goes first)
    int cur_pos = 0;                   // position of the request being served

    // What goes first has the LARGEST value.  Without a schedule: the oldest use.  With one: the position that comes up
    // last counted from the request's (a resident of the request's own position was not wanted this time round and
    // is a whole cycle away), the older use among equals.
    uint64_t evict_rank(const Resident& r) const
    {
        const uint64_t age = clock - r.tick;                 // < 2^40 in any run that finishes
        if (n_pos <= 0) return age;
        int d = (r.pos - cur_pos) % n_pos;
        if (d <= 0) d += n_pos;
        return ((uint64_t)d << 40) | (age & ((1ull << 40) - 1));
    }

    int format_of(int b) const
    {
        for (size_t i = 0; i < bits.size(); i++)
            if (bits[i] == b) return (int)i;
        return -1;
    }
    int64_t offset_of(const Resident& r) const
    {
        return (int64_t)(blocks[r.block].base + (size_t)r.slot * slot_bytes[r.fmt]);
    }
    void release(int64_t key)
    {
        auto it = where.find(key);
        Block& b = blocks[it->second.block];
        b.keys[it->second.slot] = kNoKey;
        if (--b.used == 0) b.fmt = -1;
        where.erase(it);
    }
    // a free slot of format f, or false
    bool take_free(int f, int& block, int& slot)
    {
        for (size_t i = 0; i < blocks.size(); i++) {
            Block& b = blocks[i];
            if (b.fmt != f || b.used == slots_per_block[f]) continue;
            for (int s = 0; s < slots_per_block[f]; s++)
                if (b.keys[s] == kNoKey) {
                    block = (int)i;
                    slot = s;
                    return true;
                }
        }
        for (size_t i = 0; i < blocks.size(); i++) {
            Block& b = blocks[i];
            if (b.fmt != -1 || (b.pin >= 0 && b.pin != f)) continue;
            b.fmt = f;
            b.used = 0;
            b.keys.assign((size_t)slots_per_block[f], kNoKey);
            block = (int)i;
            slot = 0;
            return true;
        }
        return false;
    }
};

extern "C" {

int dymoe_cache_create(dymoe_cache** out, size_t budget_bytes, int n_formats, const int32_t* format_bits,
                       const size_t* slot_bytes)
{
    if (!out || !format_bits || !slot_bytes) return DYMOE_EINVAL;
    if (n_formats < 1 || n_formats > DYMOE_CACHE_MAX_FORMATS) return DYMOE_EINVAL;
    dymoe_cache* c = new (std::nothrow) dymoe_cache;
    if (!c) return DYMOE_EHIP;
    size_t largest = 0;
    for (int i = 0; i < n_formats; i++) {
        const int b = format_bits[i];
        bool dup = false;
        for (int j = 0; j < i; j++) dup = dup || format_bits[j] == b;
        if (!(b == 2 || b == 4 || b == 8 || b == 16) || dup || slot_bytes[i] == 0) {
            delete c;
            return DYMOE_EINVAL;
        }
        c->bits.push_back(b);
        c->slot_bytes.push_back((slot_bytes[i] + 255) / 256 * 256);
        largest = std::max(largest, c->slot_bytes.back());
    }
    c->block_bytes = largest;
    for (int i = 0; i < n_formats; i++) {
        const size_t n = largest / c->slot_bytes[i];
        if (n > DYMOE_CACHE_MAX_EVICT) {          // an eviction is reported key by key
            delete c;
            return DYMOE_ENOTSUP;
        }
        c->slots_per_block.push_back((int)n);
    }
    const size_t n_blocks = budget_bytes / largest;
    if (n_blocks == 0) {
        delete c;
        return DYMOE_ENOSPC;
    }
    c->blocks.resize(n_blocks);
    for (size_t i = 0; i < n_blocks; i++) c->blocks[i].base = i * largest;
    *out = c;
    return DYMOE_OK;
}

int dymoe_cache_create_pools(dymoe_cache** out, int n_formats, const int32_t* format_bits, const size_t* slot_bytes,
                             const int32_t* slot_counts)
{
    if (!out || !format_bits || !slot_bytes || !slot_counts) return DYMOE_EINVAL;
    if (n_formats < 1 || n_formats > DYMOE_CACHE_MAX_FORMATS) return DYMOE_EINVAL;
    dymoe_cache* c = new (std::nothrow) dymoe_cache;
    if (!c) return DYMOE_EHIP;
    size_t total = 0, pos = 0;
    for (int i = 0; i < n_formats; i++) {
        const int b = format_bits[i];
        bool dup = false;
        for (int j = 0; j < i; j++) dup = dup || format_bits[j] == b;
        if (!(b == 2 || b == 4 || b == 8 || b == 16) || dup || slot_bytes[i] == 0 || slot_counts[i] < 1) {
            delete c;
            return DYMOE_EINVAL;
        }
        c->bits.push_back(b);
        c->slot_bytes.push_back((slot_bytes[i] + 255) / 256 * 256);
        c->slots_per_block.push_back(1);
        total += (size_t)slot_counts[i];
    }
    c->blocks.resize(total);
    size_t n = 0;
    for (int i = 0; i < n_formats; i++)
        for (int j = 0; j < slot_counts[i]; j++, n++) {
            c->blocks[n].pin = i;
            c->blocks[n].base = pos;
            pos += c->slot_bytes[i];
        }
    c->block_bytes = pos;       // the whole arena: what dymoe_cache_block_bytes reports for a fixed partition
    *out = c;
    return DYMOE_OK;
}

void dymoe_cache_destroy(dymoe_cache* c) { delete c; }

size_t dymoe_cache_block_bytes(const dymoe_cache* c) { return c ? c->block_bytes : 0; }

size_t dymoe_cache_bytes_resident(const dymoe_cache* c)
{
    if (!c) return 0;
    size_t n = 0;
    for (const auto& kv : c->where) n += c->slot_bytes[kv.second.fmt];
    return n;
}

int dymoe_cache_lookup(const dymoe_cache* c, int64_t key, int32_t* bits, int64_t* offset)
{
    if (!c) return DYMOE_EINVAL;
    auto it = c->where.find(key);
    if (it == c->where.end()) return 0;
    if (bits) *bits = c->bits[it->second.fmt];
    if (offset) *offset = c->offset_of(it->second);
    return 1;
}

int dymoe_cache_set_cyclic(dymoe_cache* c, int n_positions)
{
    if (!c || n_positions < 0) return DYMOE_EINVAL;
    c->n_pos = n_positions;
    c->cur_pos = 0;
    return DYMOE_OK;
}

int dymoe_cache_request(dymoe_cache* c, int64_t key, int want_bits, const int64_t* protect, int n_protect,
                        dymoe_cache_action* out)
{
    return dymoe_cache_request_at(c, key, want_bits, protect, n_protect, c ? c->cur_pos : 0, out);
}

int dymoe_cache_request_at(dymoe_cache* c, int64_t key, int want_bits, const int64_t* protect, int n_protect,
                           int position, dymoe_cache_action* out)
{
    if (!c || !out || n_protect < 0 || (n_protect > 0 && !protect) || key == kNoKey) return DYMOE_EINVAL;
    if (position < 0 || (c->n_pos > 0 && position >= c->n_pos)) return DYMOE_EINVAL;
    const int f = c->format_of(want_bits);
    if (f < 0) return DYMOE_EINVAL;
    c->cur_pos = position;
    out->n_evicted = 0;
    out->dropped_offset = -1;
    c->clock++;
    auto it = c->where.find(key);
    if (it != c->where.end() && c->bits[it->second.fmt] >= want_bits) {      // Conservative Reuse, or an exact hit
        it->second.tick = c->clock;
        it->second.pos = position;
        out->kind = DYMOE_CACHE_HIT;
        out->use_bits = c->bits[it->second.fmt];
        out->load_bits = 0;
        out->offset = c->offset_of(it->second);
        return DYMOE_OK;
    }
    auto is_protected = [&](int64_t k) {
        for (int i = 0; i < n_protect; i++)
            if (protect[i] == k) return true;
        return false;
    };
    int block = -1, slot = -1;
    const bool promote = it != c->where.end();
    // Room is found before anything is changed, so that a request that cannot be served leaves the cache as it was.
    if (!c->take_free(f, block, slot)) {
        // (a) the unprotected resident of the requested format that goes first (evict_rank: least recently used, or
        //     farthest next visit under a cyclic schedule)
        int64_t own = kNoKey;
        uint64_t own_rank = 0;
        for (const auto& kv : c->where)
            if (kv.second.fmt == f && kv.first != key && !is_protected(kv.first)) {
                const uint64_t rk = c->evict_rank(kv.second);
                if (own == kNoKey || rk > own_rank || (rk == own_rank && kv.first < own)) {
                    own = kv.first;
                    own_rank = rk;
                }
            }
        // (b) the block of another format without a protected resident that goes first, a block ranking with the
        //     resident of its that goes LAST (the expert being promoted does not count: its slot is released below, by
        //     the promotion itself)
        int other = -1;
        uint64_t other_rank = 0;
        for (size_t i = 0; i < c->blocks.size(); i++) {
            const Block& b = c->blocks[i];
            if (b.fmt < 0 || b.fmt == f || b.pin >= 0) continue;      // (a pinned block serves its own format only)
            uint64_t keep = UINT64_MAX;          // the smallest rank among the block's residents
            bool ok = true;
            for (int64_t k : b.keys) {
                if (k == kNoKey) continue;
                if (k != key && is_protected(k)) ok = false;
                if (k != key) keep = std::min(keep, c->evict_rank(c->where[k]));
            }
            if (ok && (other < 0 || keep > other_rank)) {
                other = (int)i;
                other_rank = keep;
            }
        }
        if (own == kNoKey && other < 0) return DYMOE_ENOSPC;
        if (own != kNoKey && (other < 0 || own_rank >= other_rank)) {
            const Resident r = c->where[own];
            out->evicted[out->n_evicted++] = own;
            c->release(own);
            block = r.block;
            slot = r.slot;
            Block& b = c->blocks[block];          // release() frees a block that became empty: claim it back
            if (b.fmt == -1) {
                b.fmt = f;
                b.keys.assign((size_t)c->slots_per_block[f], kNoKey);
            }
        } else {
            const std::vector<int64_t> keys = c->blocks[other].keys;
            for (int64_t k : keys) {
                if (k == kNoKey) continue;
                if (k == key) {                   // the lower format of the expert being promoted
                    out->dropped_offset = c->offset_of(c->where[k]);
                    c->release(k);
                    continue;
                }
                out->evicted[out->n_evicted++] = k;
                c->release(k);
            }
            Block& b = c->blocks[other];
            b.fmt = f;
            b.used = 0;
            b.keys.assign((size_t)c->slots_per_block[f], kNoKey);
            block = other;
            slot = 0;
        }
    }
    if (promote && c->where.count(key)) {                                    // Precision Promotion: the lower format goes
        out->dropped_offset = c->offset_of(c->where[key]);
        c->release(key);                          // (a slot of another format, hence of another block than the new one)
    }
    Block& b = c->blocks[block];
    b.keys[slot] = key;
    b.used++;
    Resident r{f, block, slot, c->clock, position};
    c->where[key] = r;
    out->kind = promote ? DYMOE_CACHE_PROMOTE : DYMOE_CACHE_MISS;
    out->use_bits = want_bits;
    out->load_bits = want_bits;
    out->offset = c->offset_of(r);
    return DYMOE_OK;
}

}  // extern "C"
