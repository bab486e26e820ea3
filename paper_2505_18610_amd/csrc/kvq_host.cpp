// Host side of libkvq: configuration checks, byte-budget accounting, shrink policies (Sec. 3.1), the page
// allocator over the caller's arena, device table maintenance and the C ABI declared in include/kvq.h.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cmath>
#include <cstring>
#include <new>
#include <set>
#include <limits>
#include <vector>

#include "../../include/kvq.h"
#include "kvq_internal.h"
#include "kvq_ring.h"

namespace {

constexpr int kMaxOrder = 4;  // allocation blocks of 1, 2, 4, 8, 16 units; a unit is one metadata block
constexpr int kRingSegments = 4;
constexpr uint64_t kRingSegmentBytes = 1u << 20;  // the pinned staging ring: 4 segments of 1 MiB

// Markers of the staging ring: one HIP event per segment, recorded on the cache's stream.
struct RingEvents {
    hipEvent_t ev[kRingSegments] = {};
    hipStream_t stream = nullptr;
    bool record(int i) { return hipEventRecord(ev[i], stream) == hipSuccess; }
    bool wait(int i) { return hipEventSynchronize(ev[i]) == hipSuccess; }
};

int order_of_bits(int bits) { return bits == 16 ? 4 : bits == 8 ? 3 : bits == 4 ? 2 : 1; }
bool valid_bits(int b) { return b == 16 || b == 8 || b == 4 || b == 2; }

// Buddy allocator in units.  Code blocks need 2^order units (2-bit: 2, 4-bit: 4, 8-bit: 8, 16-bit: 16),
// metadata blocks one unit, so every size is a power of two and freed space coalesces without compaction.
class Buddy {
public:
    void init(uint32_t n_super) {
        for (auto& f : free_) f.clear();
        for (uint32_t i = 0; i < n_super; ++i) free_[kMaxOrder].insert(i << kMaxOrder);
        total_ = (uint64_t)n_super << kMaxOrder;
        free_units_ = total_;
    }
    bool alloc(int order, uint32_t* off) {
        int o = order;
        while (o <= kMaxOrder && free_[o].empty()) ++o;
        if (o > kMaxOrder) return false;
        uint32_t blk = *free_[o].begin();
        free_[o].erase(free_[o].begin());
        while (o > order) {
            --o;
            free_[o].insert(blk + (1u << o));
        }
        free_units_ -= 1u << order;
        *off = blk;
        return true;
    }
    void release(uint32_t off, int order) {
        free_units_ += 1u << order;
        while (order < kMaxOrder) {
            uint32_t buddy = off ^ (1u << order);
            auto it = free_[order].find(buddy);
            if (it == free_[order].end()) break;
            free_[order].erase(it);
            off = std::min(off, buddy);
            ++order;
        }
        free_[order].insert(off);
    }
    uint64_t free_units() const { return free_units_; }

private:
    std::set<uint32_t> free_[kMaxOrder + 1];
    uint64_t total_ = 0, free_units_ = 0;
};

struct Page {
    int bits = 16;
    int n = 0;              // tokens stored
    uint32_t code_unit = 0; // allocation offsets in units
    uint32_t meta_unit = 0; // valid when the page has metadata (bits < 16, or the integer 16-bit tier)
};

struct Layer {
    uint64_t budget = 0;
    int fbit = 2;
    int T = 0;
    bool reparam = false;  // keys stored as K / lambda, queries multiplied by lambda (Sec. 3.3)
    bool poisoned = false; // an enqueue failed after the host tables had been updated: unusable until kvq_cache_reset
    std::vector<Page> pages;
    // split plan cache of kvq_decode_attention
    int plan_tiles = -1, plan_splits = 0;
    uint64_t version = 0, plan_version = ~0ull;
    int32_t split_begin[KVQ_MAX_SPLITS + 1];
};

}  // namespace

struct kvq_cache {
    kvq_config_t cfg;
    int units = 0, tpp = 0, gqa = 0, max_pages = 0;
    bool dry = false;
    uint8_t* arena = nullptr;
    uint64_t arena_bytes = 0;
    uint64_t unit_bytes = 0;
    uint64_t table_off = 0, jobs_off = 0, part_o_off = 0, part_ml_off = 0, counters_off = 0, flags_off = 0, pages_off = 0;
    uint64_t reparam_off = 0;  // per block: lambda [n_kv_heads][128] fp32, then 1 / lambda
    uint32_t* flags_dev() const { return reinterpret_cast<uint32_t*>(arena + flags_off); }
    Buddy buddy;
    std::vector<Layer> layers;
    uint8_t* ring = nullptr;
    uint8_t* ring_dev = nullptr;  // the same pinned memory as the device addresses it
    KvqStagingRing<RingEvents, kRingSegments> ring_ctl;
    RingEvents ring_events;
    bool device_ready = false;
    int splits_override = 0;
    int fused_merge = 1;
    int deterministic = 0;
    int shift_strategy = KVQ_SHIFT_EQUIVALENT;  // how 2b -> b steps treat codes, S and Z (Sec. 4.3.1)
    int tier16 = KVQ_TIER16_FP16;               // what a 16-bit token is: raw fp16, or 16-bit codes with (S, Z)
    bool int16() const { return tier16 == KVQ_TIER16_INT16; }
    bool has_meta(int bits) const { return bits < 16 || int16(); }
    int tile_cost[4] = {100, 145, 250, 300};  // relative kernel time of one 2/4/8/16-bit tile (measured)
    int target_workgroups = 256;

    uint64_t bpth(int bits) const {
        return kvq_bytes_per_token_head(bits, cfg.head_dim, cfg.group, cfg.count_metadata_in_budget, int16() ? 1 : 0);
    }
    uint64_t unit_off_bytes(uint32_t unit) const { return pages_off + (uint64_t)unit * unit_bytes; }
    KvqPageDesc desc(const Page& p) const {
        KvqPageDesc d;
        d.code_off256 = (uint32_t)(unit_off_bytes(p.code_unit) / 256);
        d.meta_off256 = has_meta(p.bits) ? (uint32_t)(unit_off_bytes(p.meta_unit) / 256) : 0u;
        d.bits = (uint32_t)p.bits;
        d.int16 = (p.bits == 16 && int16()) ? 1u : 0u;
        return d;
    }
    float* lambda_dev(int layer) const {  // lambda of the block; its reciprocals follow
        return reinterpret_cast<float*>(arena + reparam_off) + (size_t)layer * 2 * cfg.n_kv_heads * KVQ_D;
    }
    KvqPageDesc* table_dev(int layer) const {
        return reinterpret_cast<KvqPageDesc*>(arena + table_off) + (size_t)layer * max_pages;
    }
};

namespace {

struct Regions {
    uint64_t table_off, jobs_off, part_o_off, part_ml_off, counters_off, flags_off, reparam_off, pages_off;
};
uint64_t align_up(uint64_t x, uint64_t a) { return (x + a - 1) / a * a; }

bool check_config(const kvq_config_t* c) {
    if (!c) return false;
    if (c->n_layers < 1 || c->batch < 1 || c->n_kv_heads < 1 || c->n_q_heads < 1) return false;
    if (c->head_dim != KVQ_D || (c->group != 32 && c->group != 64 && c->group != 128)) return false;
    if (c->n_q_heads % c->n_kv_heads != 0 || c->n_q_heads / c->n_kv_heads > KVQ_MAX_GQA) return false;
    if (c->page_tokens < 32 || c->page_tokens % 32 != 0 || c->page_tokens > 32768) return false;
    if (c->max_tokens < 1 || c->max_tokens > (1 << 26)) return false;  // tile indices stay below 2^21 (exact magic division)
    if (c->window < 0 || c->window % c->page_tokens != 0) return false;
    if (c->n_sink < 0 || c->n_sink % c->page_tokens != 0) return false;
    if (c->policy != KVQ_POLICY_PAPER && c->policy != KVQ_POLICY_OLDEST_FIRST) return false;
    if ((int64_t)c->batch * c->n_kv_heads > 65535) return false;
    return true;
}

Regions layout_regions(const kvq_config_t* c) {
    Regions r;
    uint64_t units = (uint64_t)c->batch * c->n_kv_heads;
    uint64_t max_pages = ((uint64_t)c->max_tokens + c->page_tokens - 1) / c->page_tokens;
    uint64_t off = 0;
    r.table_off = off;     off = align_up(off + (uint64_t)c->n_layers * max_pages * sizeof(KvqPageDesc), 256);
    r.jobs_off = off;      off = align_up(off + max_pages * sizeof(KvqRequantJob), 256);
    r.part_o_off = off;    off = align_up(off + units * KVQ_MAX_SPLITS * 16 * KVQ_D * sizeof(float), 256);
    r.part_ml_off = off;   off = align_up(off + units * KVQ_MAX_SPLITS * 32 * sizeof(float), 256);
    r.counters_off = off;  off = align_up(off + units * sizeof(uint32_t), 256);
    r.flags_off = off;     off = align_up(off + 64, 256);
    r.reparam_off = off;   off = align_up(off + (uint64_t)c->n_layers * 2 * c->n_kv_heads * KVQ_D * sizeof(float), 256);
    r.pages_off = align_up(off, 4096);
    return r;
}

hipStream_t as_stream(void* s) { return static_cast<hipStream_t>(s); }

// Copy `bytes` of host data to device memory in stream order through the pinned staging ring (in pieces of at most
// one ring segment).  The host waits only if it is a whole ring ahead of the device.
kvq_status_t upload(kvq_cache* c, void* dst_dev, const void* src, uint64_t bytes, hipStream_t s) {
    c->ring_events.stream = s;
    const uint8_t* from = static_cast<const uint8_t*>(src);
    uint8_t* to = static_cast<uint8_t*>(dst_dev);
    while (bytes) {
        const uint64_t n = std::min<uint64_t>(bytes, c->ring_ctl.segment_bytes());
        const int64_t at = c->ring_ctl.reserve(c->ring_events, n, 64);
        if (at < 0) return KVQ_E_HIP;
        std::memcpy(c->ring + at, from, n);
        if (hipMemcpyAsync(to, c->ring + at, n, hipMemcpyHostToDevice, s) != hipSuccess) return KVQ_E_HIP;
        from += n; to += n; bytes -= n;
    }
    return KVQ_OK;
}

// Place `bytes` of host data (at most one ring segment) in the pinned staging ring and return where (a host address
// the device can read as well); the space is not reused before the work enqueued on s after this call has completed.
kvq_status_t stage(kvq_cache* c, const void* src, uint64_t bytes, hipStream_t s, const void** where) {
    if (bytes == 0 || bytes > c->ring_ctl.segment_bytes()) return KVQ_E_INVALID;
    c->ring_events.stream = s;
    const int64_t at = c->ring_ctl.reserve(c->ring_events, bytes, 256);
    if (at < 0) return KVQ_E_HIP;
    std::memcpy(c->ring + at, src, bytes);
    *where = c->ring_dev + at;
    return KVQ_OK;
}

kvq_status_t ensure_device(kvq_cache* c, hipStream_t s) {
    if (c->dry || c->device_ready) return KVQ_OK;
    // counters and flags are adjacent regions: one fill clears both
    if (kvq_launch_fill_u32(reinterpret_cast<uint32_t*>(c->arena + c->counters_off), 0u,
                            (size_t)((c->flags_off + 64 - c->counters_off) / sizeof(uint32_t)), s) != hipSuccess)
        return KVQ_E_HIP;
    c->device_ready = true;
    return KVQ_OK;
}

kvq_status_t upload_table(kvq_cache* c, int layer, int first, int last, hipStream_t s) {
    if (c->dry || last <= first) return KVQ_OK;
    std::vector<KvqPageDesc> d((size_t)(last - first));
    for (int i = first; i < last; ++i) d[(size_t)(i - first)] = c->desc(c->layers[(size_t)layer].pages[(size_t)i]);
    return upload(c, c->table_dev(layer) + first, d.data(), d.size() * sizeof(KvqPageDesc), s);
}

uint64_t bytes_used(const kvq_cache* c, const Layer& L) {
    uint64_t u = 0;
    for (const Page& p : L.pages) u += (uint64_t)p.n * c->units * c->bpth(p.bits);
    return u;
}

// Width of the block's bulk: smallest width among pages after the sink (16 if there is none).
int current_bits(const kvq_cache* c, const std::vector<int>& bits) {
    int first = c->cfg.n_sink / c->cfg.page_tokens, b = 16;
    for (size_t i = (size_t)first; i < bits.size(); ++i) b = std::min(b, bits[i]);
    return b;
}
int current_bits(const kvq_cache* c, const Layer& L) {
    std::vector<int> bits(L.pages.size());
    for (size_t i = 0; i < bits.size(); ++i) bits[i] = L.pages[i].bits;
    return current_bits(c, bits);
}

// Sink pages and pages overlapping the most recent `window` tokens are never lowered.
bool is_protected(const kvq_cache* c, int T, int page) {
    const int P = c->cfg.page_tokens;
    if (page < c->cfg.n_sink / P) return true;
    return c->cfg.window > 0 && (int64_t)(page + 1) * P > (int64_t)T - c->cfg.window;
}

struct Lowering {  // one page to lower and the blocks allocated for it
    int page, from, to;
    uint32_t new_code = 0, new_meta = 0;
};

// Allocate destination blocks for a set of lowerings (a metadata block too when the source page has none); on
// failure release what was taken.
bool alloc_lowerings(kvq_cache* c, std::vector<Lowering>& low) {
    for (size_t i = 0; i < low.size(); ++i) {
        bool ok = c->buddy.alloc(order_of_bits(low[i].to), &low[i].new_code);
        bool ok2 = true;
        if (ok && !c->has_meta(low[i].from)) ok2 = c->buddy.alloc(0, &low[i].new_meta);
        if (!ok || !ok2) {
            if (ok) c->buddy.release(low[i].new_code, order_of_bits(low[i].to));
            for (size_t k = 0; k < i; ++k) {
                c->buddy.release(low[k].new_code, order_of_bits(low[k].to));
                if (!c->has_meta(low[k].from)) c->buddy.release(low[k].new_meta, 0);
            }
            return false;
        }
    }
    return true;
}

// Pages of the integer 16-bit tier go down one halving at a time; raw fp16 pages reach any width in one step.
bool lowers_in_steps(const kvq_cache* c, const std::vector<Lowering>& low) {
    return !low.empty() && c->int16() && low[0].from == 16 && low[0].to < 8;
}

// Destination blocks of the first step of run_lowerings, taken ahead of it (so that a caller can find out that the
// arena is full before it changes anything), and their release when that caller gives up.  A later step of a chain
// cannot run out of blocks: each step has just freed a larger block per page than the next one takes.
bool alloc_first_step(kvq_cache* c, std::vector<Lowering>& low) {
    if (low.empty()) return true;
    const int to = low[0].to;
    const bool steps = lowers_in_steps(c, low);
    if (steps) for (auto& w : low) w.to = 8;
    const bool ok = alloc_lowerings(c, low);
    if (steps) for (auto& w : low) w.to = to;
    return ok;
}
void release_first_step(kvq_cache* c, std::vector<Lowering>& low) {
    const bool steps = lowers_in_steps(c, low);
    for (auto& w : low) {
        c->buddy.release(w.new_code, order_of_bits(steps ? 8 : w.to));
        if (!c->has_meta(w.from)) c->buddy.release(w.new_meta, 0);
    }
}

// Enqueue the kernel for lowerings that all share (from, to) -- one halving, or fp16 values to any width -- then
// commit the host tables.  allocated: the destination blocks are in `low` already.
kvq_status_t run_lowering_step(kvq_cache* c, int layer, std::vector<Lowering>& low, hipStream_t s, bool allocated = false) {
    if (low.empty()) return KVQ_OK;
    Layer& L = c->layers[(size_t)layer];
    const int from = low[0].from, to = low[0].to;
    const bool fresh_meta = !c->has_meta(from);  // raw fp16 pages carry no metadata yet
    if (!allocated && !alloc_lowerings(c, low)) return KVQ_E_OOM;
    if (!c->dry) {
        std::vector<KvqRequantJob> jobs(low.size());
        for (size_t i = 0; i < low.size(); ++i) {
            const Page& p = L.pages[(size_t)low[i].page];
            jobs[i].src_code_off256 = (uint32_t)(c->unit_off_bytes(p.code_unit) / 256);
            jobs[i].dst_code_off256 = (uint32_t)(c->unit_off_bytes(low[i].new_code) / 256);
            jobs[i].meta_off256 = (uint32_t)(c->unit_off_bytes(fresh_meta ? low[i].new_meta : p.meta_unit) / 256);
            jobs[i].n_tiles = (uint32_t)((p.n + KVQ_TILE_TOKENS - 1) / KVQ_TILE_TOKENS);
        }
        KvqRequantJob* jd = reinterpret_cast<KvqRequantJob*>(c->arena + c->jobs_off);
        const bool by_arg = jobs.size() <= (size_t)KVQ_JOBS_BY_ARG;  // short lists ride in the kernel arguments
        kvq_status_t st = by_arg ? KVQ_OK : upload(c, jd, jobs.data(), jobs.size() * sizeof(KvqRequantJob), s);
        hipError_t e = hipSuccess;
        if (st == KVQ_OK) {
            const KvqRequantJob* jh = by_arg ? jobs.data() : nullptr;
            e = fresh_meta ? kvq_launch_quant16(to, c->arena, jd, jh, (int)jobs.size(), c->tpp, c->units, c->flags_dev(), c->cfg.group, s)
                             : kvq_launch_shrink(to, c->shift_strategy, c->arena, jd, jh, (int)jobs.size(), c->tpp, c->units, c->flags_dev(), s);
        }
        if (st != KVQ_OK || e != hipSuccess) {
            for (auto& w : low) {
                c->buddy.release(w.new_code, order_of_bits(w.to));
                if (fresh_meta) c->buddy.release(w.new_meta, 0);
            }
            return st != KVQ_OK ? st : KVQ_E_HIP;
        }
    }
    int lo = (int)L.pages.size(), hi = 0;
    for (auto& w : low) {
        Page& p = L.pages[(size_t)w.page];
        c->buddy.release(p.code_unit, order_of_bits(p.bits));  // reused only by work enqueued later
        p.code_unit = w.new_code;
        if (fresh_meta) p.meta_unit = w.new_meta;
        p.bits = to;
        lo = std::min(lo, w.page);
        hi = std::max(hi, w.page + 1);
    }
    L.version++;
    const kvq_status_t up = upload_table(c, layer, lo, hi, s);
    if (up != KVQ_OK) L.poisoned = true;  // host tables and device page table disagree
    return up;
}

// Lower a set of pages that share (from, to).  Pages of the integer 16-bit tier go down one halving at a time
// (16 -> 8 -> 4 -> 2 by the configured shift strategy); raw fp16 pages are quantized to the target width directly.
// first_allocated: alloc_first_step has been called on `low`.
kvq_status_t run_lowerings(kvq_cache* c, int layer, std::vector<Lowering>& low, hipStream_t s, bool first_allocated = false) {
    if (low.empty()) return KVQ_OK;
    const int to = low[0].to;
    if (!lowers_in_steps(c, low)) return run_lowering_step(c, layer, low, s, first_allocated);
    for (int b = 8; b >= to; b /= 2) {
        const bool have = first_allocated && b == 8;
        for (auto& w : low) {
            w.from = 2 * b;
            w.to = b;
            if (!have) w.new_code = w.new_meta = 0;
        }
        kvq_status_t st = run_lowering_step(c, layer, low, s, have);
        if (st != KVQ_OK) return st;  // the pages stay at the width they reached
    }
    return KVQ_OK;
}

void build_segments(const kvq_cache* c, const Layer& L, std::vector<kvq_segment_info_t>& out) {
    const int P = c->cfg.page_tokens;
    out.clear();
    for (size_t i = 0; i < L.pages.size(); ++i) {
        int t0 = (int)i * P, t1 = t0 + L.pages[i].n;
        if (!out.empty() && out.back().bits == L.pages[i].bits) out.back().token_end = t1;
        else out.push_back(kvq_segment_info_t{t0, t1, L.pages[i].bits});
    }
}

// Relative time one tile of each width costs the attention kernel (measured on MI355X: the narrow widths are
// bound by de-quantization work, the wide ones by their bytes).
int cost_index(int bits) { return bits == 16 ? 3 : bits == 8 ? 2 : bits == 4 ? 1 : 0; }

// Cost-balanced split of the tile range.
void plan_splits(kvq_cache* c, Layer& L, int n_tiles, int n_splits) {
    if (L.plan_tiles == n_tiles && L.plan_splits == n_splits && L.plan_version == L.version) return;
    const int tpp = c->tpp;
    uint64_t total = 0;
    for (size_t i = 0; i < L.pages.size(); ++i) {
        int nt = std::min(tpp, n_tiles - (int)i * tpp);
        if (nt <= 0) break;
        int b = L.pages[i].bits;
        total += (uint64_t)nt * (uint64_t)c->tile_cost[cost_index(b)];
    }
    int sp = 1;
    L.split_begin[0] = 0;
    uint64_t cum = 0;
    for (size_t i = 0; i < L.pages.size() && sp < n_splits; ++i) {
        int nt = std::min(tpp, n_tiles - (int)i * tpp);
        if (nt <= 0) break;
        uint64_t cost = (uint64_t)c->tile_cost[cost_index(L.pages[i].bits)];
        uint64_t page_end = cum + cost * nt;
        while (sp < n_splits) {
            uint64_t target = (total * sp + n_splits - 1) / n_splits;
            if (target > page_end) break;
            uint64_t k = target <= cum ? 0 : (target - cum + cost - 1) / cost;
            if ((tpp & 1) == 0) k = std::min<uint64_t>((k + 1) & ~1ull, (uint64_t)nt);  // chunks are tile pairs
            L.split_begin[sp++] = (int)i * tpp + (int)k;
        }
        cum = page_end;
    }
    while (sp <= n_splits) L.split_begin[sp++] = n_tiles;
    L.plan_tiles = n_tiles;
    L.plan_splits = n_splits;
    L.plan_version = L.version;
}

}  // namespace

extern "C" {

uint64_t kvq_bytes_per_token_head(int32_t bits, int32_t head_dim, int32_t group, int32_t count_metadata,
                                  int32_t int16_tier) {
    if (!valid_bits(bits) || head_dim <= 0 || group <= 0) return 0;
    uint64_t n = 2ull * head_dim * bits / 8;
    if (count_metadata && (bits < 16 || int16_tier)) n += 2ull * (head_dim / group) * 4;
    return n;
}

uint64_t kvq_arena_bytes(const kvq_config_t* cfg, uint64_t payload_bytes) {
    if (!check_config(cfg)) return 0;
    Regions r = layout_regions(cfg);
    uint64_t super = (32ull * cfg->page_tokens * cfg->batch * cfg->n_kv_heads) << kMaxOrder;
    return r.pages_off + align_up(payload_bytes, super);
}

kvq_status_t kvq_cache_create(const kvq_config_t* cfg, const uint64_t* block_budget_bytes_host,
                              const uint8_t* block_fbit_host, void* arena_dev, uint64_t arena_bytes,
                              kvq_cache_t** out) {
    if (!out) return KVQ_E_INVALID;
    *out = nullptr;
    if (!check_config(cfg) || !block_budget_bytes_host || !block_fbit_host) return KVQ_E_INVALID;
    for (int i = 0; i < cfg->n_layers; ++i)
        if (!valid_bits(block_fbit_host[i])) return KVQ_E_INVALID;
    if (arena_dev && (reinterpret_cast<uintptr_t>(arena_dev) & 255u)) return KVQ_E_INVALID;
    kvq_cache* c = new (std::nothrow) kvq_cache();
    if (!c) return KVQ_E_OOM;
    c->cfg = *cfg;
    c->units = cfg->batch * cfg->n_kv_heads;
    c->tpp = cfg->page_tokens / KVQ_TILE_TOKENS;
    c->gqa = cfg->n_q_heads / cfg->n_kv_heads;
    c->max_pages = (cfg->max_tokens + cfg->page_tokens - 1) / cfg->page_tokens;
    c->dry = (arena_dev == nullptr);
    c->arena = static_cast<uint8_t*>(arena_dev);
    c->arena_bytes = arena_bytes;
    c->unit_bytes = 32ull * cfg->page_tokens * c->units;
    Regions r = layout_regions(cfg);
    c->table_off = r.table_off; c->jobs_off = r.jobs_off; c->part_o_off = r.part_o_off;
    c->part_ml_off = r.part_ml_off; c->counters_off = r.counters_off; c->flags_off = r.flags_off; c->pages_off = r.pages_off;
    c->reparam_off = r.reparam_off;
    uint64_t super = c->unit_bytes << kMaxOrder;
    if (arena_bytes < c->pages_off + super) { delete c; return KVQ_E_OOM; }
    uint64_t n_super = (arena_bytes - c->pages_off) / super;
    if ((c->pages_off + n_super * super) / 256 > 0xffffffffull) { delete c; return KVQ_E_INVALID; }
    c->buddy.init((uint32_t)n_super);
    c->layers.resize((size_t)cfg->n_layers);
    for (int i = 0; i < cfg->n_layers; ++i) {
        c->layers[(size_t)i].budget = block_budget_bytes_host[i];
        c->layers[(size_t)i].fbit = block_fbit_host[i];
    }
    if (!c->dry) {
        c->ring_ctl.init(kRingSegmentBytes);
        if (hipHostMalloc(reinterpret_cast<void**>(&c->ring), c->ring_ctl.total_bytes(), hipHostMallocDefault) != hipSuccess) {
            delete c;
            return KVQ_E_HIP;
        }
        for (int i = 0; i < kRingSegments; ++i) {
            if (hipEventCreateWithFlags(&c->ring_events.ev[i], hipEventDisableTiming) != hipSuccess) {
                for (int k = 0; k < i; ++k) (void)hipEventDestroy(c->ring_events.ev[k]);
                (void)hipHostFree(c->ring);
                delete c;
                return KVQ_E_HIP;
            }
        }
        if (hipHostGetDevicePointer(reinterpret_cast<void**>(&c->ring_dev), c->ring, 0) != hipSuccess) {
            for (int i = 0; i < kRingSegments; ++i) (void)hipEventDestroy(c->ring_events.ev[i]);
            (void)hipHostFree(c->ring);
            delete c;
            return KVQ_E_HIP;
        }
        int dev = 0;
        hipDeviceProp_t prop;
        if (hipGetDevice(&dev) == hipSuccess && hipGetDeviceProperties(&prop, dev) == hipSuccess &&
            prop.multiProcessorCount > 0)
            c->target_workgroups = prop.multiProcessorCount;  // one 8-wavefront workgroup per compute unit
    }
    *out = c;
    return KVQ_OK;
}

void kvq_cache_destroy(kvq_cache_t* c) {
    if (!c) return;
    if (c->ring) {
        (void)hipHostFree(c->ring);
        for (int i = 0; i < kRingSegments; ++i) (void)hipEventDestroy(c->ring_events.ev[i]);
    }
    delete c;
}

}  // extern "C"

namespace {

// What a deferred single-token append into the 16-bit tier leaves for the attention launch to do.
struct DeferredAppend {
    bool int16_too = false;  // in: the attention launch that follows can also append into the integer 16-bit tier
    bool active = false;
    int t_old = 0;
    KvqPageDesc desc{};
};

// Bookkeeping of an append, worked out without touching the cache: entry width, page widths and fill counts
// afterwards, the window pages the append evicts and the width they go to.
struct AppendPlan {
    int e = 16, T = 0, bcur = 16;
    std::vector<int> bits, cnt, evicted;
};

kvq_status_t plan_append(const kvq_cache_t* c, int32_t layer, int32_t n_new, int32_t entry_bits, AppendPlan& pl) {
    const Layer& L = c->layers[(size_t)layer];
    const kvq_config_t& cfg = c->cfg;
    const int P = cfg.page_tokens;
    if (L.poisoned) return KVQ_E_STATE;
    if ((int64_t)L.T + n_new > cfg.max_tokens) return KVQ_E_STATE;
    int e = entry_bits;
    if (e == 0) e = (cfg.policy == KVQ_POLICY_OLDEST_FIRST || cfg.window > 0) ? 16 : current_bits(c, L);
    if (L.T % P != 0 && L.pages.back().bits != e) return KVQ_E_STATE;
    const bool evict = entry_bits == 0 && cfg.policy == KVQ_POLICY_PAPER && cfg.window > 0;
    pl.e = e;
    pl.bits.resize(L.pages.size());
    pl.cnt.resize(L.pages.size());
    for (size_t i = 0; i < L.pages.size(); ++i) { pl.bits[i] = L.pages[i].bits; pl.cnt[i] = L.pages[i].n; }
    int T = L.T, left = n_new;
    while (left) {
        if (T % P == 0) { pl.bits.push_back(e); pl.cnt.push_back(0); }
        int take = std::min(left, P - pl.cnt.back());
        pl.cnt.back() += take; T += take; left -= take;
    }
    pl.T = T;
    pl.evicted.clear();
    pl.bcur = 16;
    if (evict) {
        pl.bcur = current_bits(c, pl.bits);
        if (pl.bcur < 16) {
            for (;;) {
                int i = (int)pl.bits.size(), first = cfg.n_sink / P;
                while (i > first && pl.bits[(size_t)i - 1] == 16) --i;  // start of the trailing 16-bit run
                if (i < (int)pl.bits.size() && T - i * P >= cfg.window + P) { pl.bits[(size_t)i] = pl.bcur; pl.evicted.push_back(i); }
                else break;
            }
        }
    }
    uint64_t used = 0;
    for (size_t i = 0; i < pl.bits.size(); ++i) used += (uint64_t)pl.cnt[i] * c->units * c->bpth(pl.bits[i]);
    if (used > L.budget) return KVQ_E_BUDGET;
    return KVQ_OK;
}

bool append_args_ok(const kvq_cache_t* c, int32_t layer, const void* k_dev, const void* v_dev, int32_t n_new,
                    int32_t entry_bits) {
    if (!c || layer < 0 || layer >= c->cfg.n_layers || n_new < 0 || n_new >= KVQ_MAX_APPEND_TOKENS) return false;
    if (entry_bits != 0 && !valid_bits(entry_bits)) return false;
    if (n_new > 0 && !c->dry && (!k_dev || !v_dev)) return false;
    return true;
}

// Carries a planned append out.  defer != nullptr: a one-token append into the 16-bit tier is not launched but
// described in *defer (page allocation, table upload and window evictions happen as usual).
kvq_status_t commit_append(kvq_cache_t* c, int32_t layer, const AppendPlan& pl, const void* k_dev, const void* v_dev,
                           int32_t n_new, const float* cos_sin_dev, hipStream_t s, DeferredAppend* defer) {
    Layer& L = c->layers[(size_t)layer];
    const int P = c->cfg.page_tokens, e = pl.e;
    // allocate the new pages
    const size_t old_pages = L.pages.size();
    std::vector<Page> fresh;
    for (size_t i = old_pages; i < pl.bits.size(); ++i) {
        Page p;
        p.bits = e;
        bool ok = c->buddy.alloc(order_of_bits(e), &p.code_unit);
        bool ok2 = true;
        if (ok && c->has_meta(e)) ok2 = c->buddy.alloc(0, &p.meta_unit);
        if (!ok || !ok2) {
            if (ok) c->buddy.release(p.code_unit, order_of_bits(e));
            for (Page& q : fresh) {
                c->buddy.release(q.code_unit, order_of_bits(e));
                if (c->has_meta(e)) c->buddy.release(q.meta_unit, 0);
            }
            return KVQ_E_OOM;
        }
        fresh.push_back(p);
    }
    auto release_fresh = [&]() {
        for (Page& q : fresh) {
            c->buddy.release(q.code_unit, order_of_bits(e));
            if (c->has_meta(e)) c->buddy.release(q.meta_unit, 0);
        }
    };
    // pages that leave the window in this call are lowered behind the append: their destination blocks are taken now,
    // while a full arena can still be reported with nothing changed
    std::vector<Lowering> low;
    for (int i : pl.evicted) low.push_back(Lowering{i, 16, pl.bcur});
    if (!alloc_first_step(c, low)) {
        release_fresh();
        return KVQ_E_OOM;
    }
    kvq_status_t st = ensure_device(c, s);
    if (st != KVQ_OK) {
        release_first_step(c, low);
        release_fresh();
        return st;
    }
    const int t_old = L.T, T = pl.T;
    for (Page& p : fresh) L.pages.push_back(p);
    for (size_t i = 0; i < L.pages.size(); ++i) L.pages[i].n = pl.cnt[i];
    L.T = T;
    L.version++;
    // From here on the host tables count the new tokens: a failing enqueue leaves the block unusable (poisoned).
    st = upload_table(c, layer, (int)old_pages, (int)L.pages.size(), s);
    if (st != KVQ_OK) {
        release_first_step(c, low);
        L.poisoned = true;
        return st;
    }
    if (!c->dry && defer && n_new == 1 && e == 16 && (!c->int16() || defer->int16_too)) {
        defer->active = true;
        defer->t_old = t_old;
        defer->desc = c->desc(L.pages[(size_t)(t_old / P)]);
    } else if (!c->dry) {
        // short appends (at most two pages touched) carry the page descriptors in the kernel arguments
        const int pg0 = t_old / P, pg1 = (T - 1) / P;
        KvqPageDesc two[2];
        const bool by_arg = pg1 - pg0 <= 1;
        if (by_arg) {
            two[0] = c->desc(L.pages[(size_t)pg0]);
            two[1] = c->desc(L.pages[(size_t)pg1]);
        }
        if (kvq_launch_append(e, c->arena, c->table_dev(layer), k_dev, v_dev, t_old, n_new, c->tpp, c->units,
                              by_arg ? two : nullptr, pg0, c->flags_dev(), c->cfg.group,
                              L.reparam ? c->lambda_dev(layer) + c->cfg.n_kv_heads * KVQ_D : nullptr, c->cfg.n_kv_heads,
                              cos_sin_dev, c->int16(), s) != hipSuccess) {
            release_first_step(c, low);
            L.poisoned = true;
            return KVQ_E_HIP;
        }
    }
    if (!low.empty()) {
        st = run_lowerings(c, layer, low, s, true);
        if (st != KVQ_OK) { L.poisoned = true; return st; }  // the plan counted these pages at their new width
    }
    return KVQ_OK;
}

kvq_status_t append_impl(kvq_cache_t* c, int32_t layer, const void* k_dev, const void* v_dev, int32_t n_new,
                         int32_t entry_bits, const float* cos_sin_dev, void* hip_stream, DeferredAppend* defer) {
    if (!append_args_ok(c, layer, k_dev, v_dev, n_new, entry_bits)) return KVQ_E_INVALID;
    if (n_new == 0) return KVQ_OK;
    AppendPlan pl;
    kvq_status_t st = plan_append(c, layer, n_new, entry_bits, pl);
    if (st != KVQ_OK) return st;
    return commit_append(c, layer, pl, k_dev, v_dev, n_new, cos_sin_dev, as_stream(hip_stream), defer);
}

}  // namespace

extern "C" {

kvq_status_t kvq_quantize_append(kvq_cache_t* c, int32_t layer, const void* k_dev, const void* v_dev,
                                 int32_t n_new, int32_t entry_bits, void* hip_stream) {
    return append_impl(c, layer, k_dev, v_dev, n_new, entry_bits, nullptr, hip_stream, nullptr);
}

kvq_status_t kvq_quantize_append_rope(kvq_cache_t* c, int32_t layer, const void* k_dev, const void* v_dev,
                                      int32_t n_new, int32_t entry_bits, const float* cos_sin_dev, void* hip_stream) {
    return append_impl(c, layer, k_dev, v_dev, n_new, entry_bits, cos_sin_dev, hip_stream, nullptr);
}

kvq_status_t kvq_progressive_requant(kvq_cache_t* c, int32_t layer, int32_t segment, int32_t reserve_tokens,
                                     void* hip_stream, int32_t* n_pages_done) {
    if (n_pages_done) *n_pages_done = 0;
    if (!c || layer < 0 || layer >= c->cfg.n_layers || segment < -1 || reserve_tokens < 0) return KVQ_E_INVALID;
    Layer& L = c->layers[(size_t)layer];
    const kvq_config_t& cfg = c->cfg;
    const int P = cfg.page_tokens;
    if (L.poisoned) return KVQ_E_STATE;
    hipStream_t s = as_stream(hip_stream);
    kvq_status_t st = ensure_device(c, s);
    if (st != KVQ_OK) return st;

    if (segment >= 0) {
        std::vector<kvq_segment_info_t> segs;
        build_segments(c, L, segs);
        if (segment >= (int)segs.size()) return KVQ_E_STATE;
        const kvq_segment_info_t sg = segs[(size_t)segment];
        if (sg.bits == 2) return KVQ_E_STATE;
        // A run that ends in the partly filled last page: lowering it would leave that page at a width other than the
        // one the policy appends at (16 bits under OLDEST_FIRST or with a window), and no token could follow.
        if (sg.token_end == L.T && L.T % P != 0 && (cfg.policy == KVQ_POLICY_OLDEST_FIRST || cfg.window > 0))
            return KVQ_E_STATE;
        std::vector<Lowering> low;
        for (int i = sg.token_begin / P; i < (sg.token_end + P - 1) / P; ++i) low.push_back(Lowering{i, sg.bits, sg.bits / 2});
        st = run_lowerings(c, layer, low, s);
        if (st == KVQ_OK && n_pages_done) *n_pages_done = (int32_t)low.size();
        return st;
    }
    if (cfg.policy == KVQ_POLICY_PAPER) {
        const int bcur = current_bits(c, L);
        if (bcur <= L.fbit) return KVQ_E_BUDGET;
        std::vector<Lowering> low;
        for (int i = 0; i < (int)L.pages.size(); ++i)
            if (L.pages[(size_t)i].bits == bcur && !is_protected(c, L.T, i)) low.push_back(Lowering{i, bcur, bcur / 2});
        if (low.empty()) return KVQ_E_BUDGET;
        st = run_lowerings(c, layer, low, s);
        if (st == KVQ_OK && n_pages_done) *n_pages_done = (int32_t)low.size();
        return st;
    }
    // OLDEST_FIRST
    const uint64_t need = (uint64_t)reserve_tokens * c->units * c->bpth(16);
    int done = 0;
    while (bytes_used(c, L) + need > L.budget) {
        int pick = -1;
        for (int i = cfg.n_sink / P; i < (int)L.pages.size(); ++i) {
            const Page& p = L.pages[(size_t)i];
            if (p.bits > L.fbit && p.n == P && (int64_t)(i + 1) * P <= (int64_t)L.T - cfg.window) { pick = i; break; }
        }
        if (pick < 0) { if (n_pages_done) *n_pages_done = done; return KVQ_E_BUDGET; }
        std::vector<Lowering> low{Lowering{pick, L.pages[(size_t)pick].bits, L.pages[(size_t)pick].bits / 2}};
        st = run_lowerings(c, layer, low, s);
        if (st != KVQ_OK) { if (n_pages_done) *n_pages_done = done; return st; }
        ++done;
    }
    if (n_pages_done) *n_pages_done = done;
    return KVQ_OK;
}

}  // extern "C"

namespace {

// Relative time the attention kernel needs for the block's tiles, and how many of them are 2 bits wide.
void tile_census(const kvq_cache_t* c, const Layer& L, int n_tiles, int* n2, int* n_all, uint64_t* cost) {
    *n2 = *n_all = 0;
    *cost = 0;
    for (size_t i = 0; i < L.pages.size(); ++i) {
        const int nt = std::min(c->tpp, n_tiles - (int)i * c->tpp);
        if (nt <= 0) break;
        *n_all += nt;
        if (L.pages[i].bits == 2) *n2 += nt;
        *cost += (uint64_t)nt * (uint64_t)c->tile_cost[cost_index(L.pages[i].bits)];
    }
}

// Fills the parameter block of one attention launch over block `layer`.  wgs_share > 0: the number of workgroups this
// cache may use (its share of a ragged batch); 0: the whole device.
kvq_status_t fill_attn_params(kvq_cache_t* c, int32_t layer, const void* q_dev, void* out_dev, int32_t out_is_fp32,
                              float softmax_scale, const DeferredAppend* app, const void* k_new, const void* v_new,
                              const float* cos_sin_dev, int wgs_share, KvqAttnParams& p) {
    if (!c || layer < 0 || layer >= c->cfg.n_layers || !q_dev || !out_dev) return KVQ_E_INVALID;
    if (c->dry) return KVQ_E_STATE;
    Layer& L = c->layers[(size_t)layer];
    if (L.T == 0 || L.poisoned) return KVQ_E_STATE;
    const int n_tiles = (L.T + KVQ_TILE_TOKENS - 1) / KVQ_TILE_TOKENS;
    int n_splits = c->splits_override;
    if (n_splits <= 0) {
        // One workgroup per compute unit when a good part of the tiles is 2 bits wide (those are bound by vector
        // issue and want every unit).  A block of wider tiles is bound by HBM, and there three quarters of the
        // units stream measurably faster than all of them (4 to 7 % on 4-, 8- and 16-bit blocks).
        int wgs = wgs_share;
        if (wgs <= 0) {
            int n2 = 0, n_all = 0;
            uint64_t cost = 0;
            tile_census(c, L, n_tiles, &n2, &n_all, &cost);
            wgs = c->target_workgroups;
            if (4 * n2 < n_all) wgs = std::max(c->units, wgs * 3 / 4);
        }
        n_splits = std::min(wgs / std::max(1, c->units), (n_tiles + 15) / 16);
    }
    n_splits = std::max(1, std::min(n_splits, std::min(KVQ_MAX_SPLITS, n_tiles)));
    plan_splits(c, L, n_tiles, n_splits);

    p.arena = c->arena;
    p.table = c->table_dev(layer);
    p.q = q_dev;
    p.lambda = L.reparam ? c->lambda_dev(layer) : nullptr;
    p.out = out_dev;
    p.part_o = reinterpret_cast<float*>(c->arena + c->part_o_off);
    p.part_ml = reinterpret_cast<float*>(c->arena + c->part_ml_off);
    p.counters = reinterpret_cast<uint32_t*>(c->arena + c->counters_off);
    p.flags = c->flags_dev();
    p.n_tokens = L.T;
    p.tiles_per_page = c->tpp;
    p.tpp_magic = c->tpp > 1 ? (uint32_t)(((1ull << 32) + (uint64_t)c->tpp - 1) / (uint64_t)c->tpp) : 0u;
    p.gqa = c->gqa;
    p.n_q_heads = c->cfg.n_q_heads;
    p.n_kv_heads = c->cfg.n_kv_heads;
    p.n_splits = n_splits;
    p.out_fp32 = out_is_fp32 ? 1 : 0;
    p.fused_merge = c->fused_merge;
    p.deterministic = c->deterministic;
    p.int16_tier = c->int16() ? 1 : 0;
    const float scale = softmax_scale != 0.f ? softmax_scale : 1.0f / std::sqrt((float)c->cfg.head_dim);
    p.scale_log2 = scale * 1.44269504088896340736f;
    std::memcpy(p.split_begin, L.split_begin, sizeof(int32_t) * (size_t)(n_splits + 1));
    for (int i = n_splits + 1; i <= KVQ_MAX_SPLITS; ++i) p.split_begin[i] = n_tiles;
    p.app_t_old = -1;
    p.app_desc = KvqPageDesc{0, 0, 0, 0};
    p.app_k = p.app_v = nullptr;
    p.app_rope = p.app_rinv = nullptr;
    if (app && app->active) {
        p.app_t_old = app->t_old;
        p.app_desc = app->desc;
        p.app_k = k_new;
        p.app_v = v_new;
        p.app_rope = cos_sin_dev;
        p.app_rinv = L.reparam ? c->lambda_dev(layer) + c->cfg.n_kv_heads * KVQ_D : nullptr;
    }
    p.app_gspan = c->cfg.group / 32;
    return KVQ_OK;
}

kvq_status_t attention_impl(kvq_cache_t* c, int32_t layer, const void* q_dev, void* out_dev, int32_t out_is_fp32,
                            float softmax_scale, void* hip_stream, const DeferredAppend* app, const void* k_new,
                            const void* v_new, const float* cos_sin_dev) {
    KvqAttnParams p;
    kvq_status_t st = fill_attn_params(c, layer, q_dev, out_dev, out_is_fp32, softmax_scale, app, k_new, v_new,
                                       cos_sin_dev, 0, p);
    if (st != KVQ_OK) return st;
    return kvq_launch_attention(p, c->units, as_stream(hip_stream)) == hipSuccess ? KVQ_OK : KVQ_E_HIP;
}

// One attention launch over block `layer` of n caches, optionally with each cache's one-token append in front.
kvq_status_t batch_impl(kvq_cache_t* const* caches, int32_t n, int32_t layer, const void* const* k_dev,
                        const void* const* v_dev, const float* const* cos_sin_dev, const void* const* q_dev,
                        void* const* out_dev, int32_t out_is_fp32, float softmax_scale, void* hip_stream, bool append) {
    if (!caches || n < 1 || n > KVQ_MAX_BATCH_CACHES || !q_dev || !out_dev) return KVQ_E_INVALID;
    if (append && (!k_dev || !v_dev)) return KVQ_E_INVALID;
    for (int i = 0; i < n; ++i) {
        kvq_cache_t* c = caches[i];
        if (!c || layer < 0 || layer >= c->cfg.n_layers || !q_dev[i] || !out_dev[i]) return KVQ_E_INVALID;
        if (append && (!k_dev[i] || !v_dev[i])) return KVQ_E_INVALID;
        if (c->dry) return KVQ_E_STATE;
        if (c->int16() != caches[0]->int16()) return KVQ_E_INVALID;  // one kernel serves one kind of 16-bit tier
        for (int k = 0; k < i; ++k)
            if (caches[k] == c) return KVQ_E_INVALID;
    }
    hipStream_t s = as_stream(hip_stream);
    std::vector<DeferredAppend> app((size_t)n);
    if (append) {
        // all or nothing as far as the bookkeeping can tell: plan every append before the first one is carried out
        std::vector<AppendPlan> plans((size_t)n);
        for (int i = 0; i < n; ++i) {
            kvq_status_t st = plan_append(caches[i], layer, 1, 0, plans[(size_t)i]);
            if (st != KVQ_OK) return st;
        }
        for (int i = 0; i < n; ++i) {
            kvq_status_t st = commit_append(caches[i], layer, plans[(size_t)i], k_dev[i], v_dev[i], 1,
                                            cos_sin_dev ? cos_sin_dev[i] : nullptr, s, &app[(size_t)i]);
            if (st != KVQ_OK) return st;
        }
    }
    // The device's workgroups are dealt to the caches so that the most loaded workgroup is as light as possible:
    // every cache starts with one split per (sequence, KV head); the cache whose workgroups carry the most tile
    // time gets one more split, as long as the workgroups last (and its splits keep 16 tiles or more).
    std::vector<uint64_t> cost((size_t)n);  // tile time of one (sequence, KV head) of the cache
    std::vector<int> splits((size_t)n, 1), max_splits((size_t)n);
    int used = 0;
    for (int i = 0; i < n; ++i) {
        kvq_cache_t* c = caches[i];
        const Layer& L = c->layers[(size_t)layer];
        if (L.T == 0) return KVQ_E_STATE;
        const int n_tiles = (L.T + KVQ_TILE_TOKENS - 1) / KVQ_TILE_TOKENS;
        int a = 0, b = 0;
        tile_census(c, L, n_tiles, &a, &b, &cost[(size_t)i]);
        max_splits[(size_t)i] = std::max(1, std::min(KVQ_MAX_SPLITS, (n_tiles + 15) / 16));
        used += c->units;
    }
    // (every compute unit is used: with ranges of unequal length the heaviest workgroup decides the launch time,
    //  which outweighs the few percent a block of equal ranges gains from leaving a quarter of the units idle)
    const int wgs = caches[0]->target_workgroups;
    for (;;) {
        int pick = -1;
        uint64_t worst = 0;
        for (int i = 0; i < n; ++i) {
            if (splits[(size_t)i] >= max_splits[(size_t)i] || used + caches[i]->units > wgs) continue;
            const uint64_t per_wg = cost[(size_t)i] / (uint64_t)splits[(size_t)i];
            if (per_wg > worst) { worst = per_wg; pick = i; }
        }
        if (pick < 0) break;
        // stop once a heavier cache could still be split but no longer fits into the workgroups that are left:
        // more splits elsewhere would not lighten the heaviest workgroup, only add merge work
        bool blocked = false;
        for (int i = 0; i < n; ++i)
            if (i != pick && cost[(size_t)i] / (uint64_t)splits[(size_t)i] > worst &&
                splits[(size_t)i] < max_splits[(size_t)i])
                blocked = true;
        if (blocked) break;
        splits[(size_t)pick]++;
        used += caches[pick]->units;
    }
    std::vector<KvqAttnParams> params((size_t)n);
    for (int i = 0; i < n; ++i) {
        kvq_status_t st = fill_attn_params(caches[i], layer, q_dev[i], out_dev[i], out_is_fp32, softmax_scale,
                                           &app[(size_t)i], append ? k_dev[i] : nullptr, append ? v_dev[i] : nullptr,
                                           cos_sin_dev ? cos_sin_dev[i] : nullptr, splits[(size_t)i] * caches[i]->units,
                                           params[(size_t)i]);
        if (st != KVQ_OK) return st;
    }
    // The kernel reads the parameter blocks straight from the pinned staging ring of the first cache (host memory the
    // device can address): a copy into the arena would be a separate transfer between two kernels on the stream, which
    // costs more than the workgroups' first reads travelling over the host link.
    kvq_cache_t* lead = caches[0];
    const KvqAttnParams* params_dev = nullptr;
    kvq_status_t st = stage(lead, params.data(), params.size() * sizeof(KvqAttnParams), s,
                            reinterpret_cast<const void**>(&params_dev));
    if (st != KVQ_OK) return st;
    std::vector<int> units((size_t)n);
    for (int i = 0; i < n; ++i) units[(size_t)i] = caches[i]->units;
    return kvq_launch_attention_batch(params_dev, params.data(), units.data(), n, s) == hipSuccess ? KVQ_OK : KVQ_E_HIP;
}

}  // namespace

extern "C" {

kvq_status_t kvq_decode_attention(kvq_cache_t* c, int32_t layer, const void* q_dev, void* out_dev,
                                  int32_t out_is_fp32, float softmax_scale, void* hip_stream) {
    return attention_impl(c, layer, q_dev, out_dev, out_is_fp32, softmax_scale, hip_stream, nullptr, nullptr, nullptr,
                          nullptr);
}

kvq_status_t kvq_decode_attention_static(kvq_cache_t* c, int32_t layer, const void* q_dev, void* out_dev,
                                         int32_t out_is_fp32, float softmax_scale, void* hip_stream) {
    KvqAttnParams p;
    kvq_status_t st = fill_attn_params(c, layer, q_dev, out_dev, out_is_fp32, softmax_scale, nullptr, nullptr, nullptr,
                                       nullptr, 0, p);
    if (st != KVQ_OK) return st;
    if (c->units > KVQ_STATIC_MAX_UNITS || (int64_t)c->units * p.n_splits > KVQ_STATIC_MAX_WGS) return KVQ_E_LIMIT;
    unsigned char* scr = nullptr;
    if (kvq_static_scratch(&scr) != hipSuccess) return KVQ_E_HIP;
    hipStream_t s = as_stream(hip_stream);
    p.part_o = reinterpret_cast<float*>(scr);
    p.part_ml = reinterpret_cast<float*>(scr + KVQ_STATIC_PART_O_BYTES);
    p.counters = reinterpret_cast<uint32_t*>(scr + KVQ_STATIC_PART_O_BYTES + KVQ_STATIC_PART_ML_BYTES);
    // The array keeps what the last call left.  Partials are written before they are read; the arrival counters must
    // start at zero (a kernel leaves them there, but a launch that failed half-way would not): a fill kernel, which a
    // caller may also capture into a graph.
    if (p.n_splits > 1 && p.fused_merge &&
        kvq_launch_fill_u32(p.counters, 0u, (size_t)c->units, s) != hipSuccess)
        return KVQ_E_HIP;
    return kvq_launch_attention(p, c->units, s) == hipSuccess ? KVQ_OK : KVQ_E_HIP;
}

kvq_status_t kvq_append_decode_attention(kvq_cache_t* c, int32_t layer, const void* k_dev, const void* v_dev,
                                         const float* cos_sin_dev, const void* q_dev, void* out_dev,
                                         int32_t out_is_fp32, float softmax_scale, void* hip_stream) {
    if (!q_dev || !out_dev) return KVQ_E_INVALID;  // nothing may be appended when the attention cannot follow
    if (c && c->dry) return KVQ_E_STATE;
    DeferredAppend app;
    app.int16_too = true;
    kvq_status_t st = append_impl(c, layer, k_dev, v_dev, 1, 0, cos_sin_dev, hip_stream, &app);
    if (st != KVQ_OK) return st;
    return attention_impl(c, layer, q_dev, out_dev, out_is_fp32, softmax_scale, hip_stream, &app, k_dev, v_dev, cos_sin_dev);
}

kvq_status_t kvq_decode_attention_batch(kvq_cache_t* const* caches, int32_t n_caches, int32_t layer,
                                        const void* const* q_dev, void* const* out_dev, int32_t out_is_fp32,
                                        float softmax_scale, void* hip_stream) {
    return batch_impl(caches, n_caches, layer, nullptr, nullptr, nullptr, q_dev, out_dev, out_is_fp32, softmax_scale,
                      hip_stream, false);
}

kvq_status_t kvq_append_decode_attention_batch(kvq_cache_t* const* caches, int32_t n_caches, int32_t layer,
                                               const void* const* k_dev, const void* const* v_dev,
                                               const float* const* cos_sin_dev, const void* const* q_dev,
                                               void* const* out_dev, int32_t out_is_fp32, float softmax_scale,
                                               void* hip_stream) {
    return batch_impl(caches, n_caches, layer, k_dev, v_dev, cos_sin_dev, q_dev, out_dev, out_is_fp32, softmax_scale,
                      hip_stream, true);
}

kvq_status_t kvq_cache_describe(const kvq_cache_t* c, int32_t layer, kvq_segment_info_t* segs_host, int32_t cap,
                                int32_t* n, uint64_t* bytes_used_out, int32_t* n_tokens, int32_t* current_bits_out) {
    if (!c || layer < 0 || layer >= c->cfg.n_layers || cap < 0 || (cap > 0 && !segs_host)) return KVQ_E_INVALID;
    const Layer& L = c->layers[(size_t)layer];
    std::vector<kvq_segment_info_t> segs;
    build_segments(c, L, segs);
    for (int i = 0; i < std::min<int>(cap, (int)segs.size()); ++i) segs_host[i] = segs[(size_t)i];
    if (n) *n = (int32_t)segs.size();
    if (bytes_used_out) *bytes_used_out = bytes_used(c, L);
    if (n_tokens) *n_tokens = L.T;
    if (current_bits_out) *current_bits_out = current_bits(c, L);
    return KVQ_OK;
}

kvq_status_t kvq_cache_export_segment(kvq_cache_t* c, int32_t layer, int32_t segment, int32_t which,
                                      void* codes_host, void* scales_host, void* zeros_host, void* hip_stream) {
    if (!c || layer < 0 || layer >= c->cfg.n_layers || segment < 0 || !codes_host) return KVQ_E_INVALID;
    if (which != KVQ_WHICH_K && which != KVQ_WHICH_V) return KVQ_E_INVALID;
    if (c->dry) return KVQ_E_STATE;
    const Layer& L = c->layers[(size_t)layer];
    if (L.poisoned) return KVQ_E_STATE;
    std::vector<kvq_segment_info_t> segs;
    build_segments(c, L, segs);
    if (segment >= (int)segs.size()) return KVQ_E_STATE;
    const kvq_segment_info_t sg = segs[(size_t)segment];
    const int b = sg.bits, P = c->cfg.page_tokens, tpp = c->tpp;
    const bool meta_out = c->has_meta(b), planes = b == 16 && c->int16();
    if (meta_out && (!scales_host || !zeros_host)) return KVQ_E_INVALID;
    hipStream_t s = as_stream(hip_stream);
    const int n_seg = sg.token_end - sg.token_begin;
    const size_t row_bytes = (size_t)KVQ_D * b / 8;
    const size_t code_block = (size_t)c->unit_bytes * b;
    std::vector<uint8_t> code(code_block), meta(meta_out ? (size_t)c->unit_bytes : 0);
    uint8_t* oc = static_cast<uint8_t*>(codes_host);
    uint16_t* os = static_cast<uint16_t*>(scales_host);
    uint16_t* oz = static_cast<uint16_t*>(zeros_host);
    for (int pg = sg.token_begin / P; pg < (sg.token_end + P - 1) / P; ++pg) {
        const Page& p = L.pages[(size_t)pg];
        if (hipMemcpyAsync(code.data(), c->arena + c->unit_off_bytes(p.code_unit), code_block, hipMemcpyDeviceToHost, s) != hipSuccess)
            return KVQ_E_HIP;
        if (meta_out && hipMemcpyAsync(meta.data(), c->arena + c->unit_off_bytes(p.meta_unit), meta.size(), hipMemcpyDeviceToHost, s) != hipSuccess)
            return KVQ_E_HIP;
        if (hipStreamSynchronize(s) != hipSuccess) return KVQ_E_HIP;
        for (int u = 0; u < c->units; ++u) {
            for (int tl = 0; tl < p.n; ++tl) {
                const int tip = tl / KVQ_TILE_TOKENS, t = tl % KVQ_TILE_TOKENS;
                const size_t tslot = (size_t)u * tpp + tip;
                const uint8_t* tile = code.data() + (tslot * 2 + (size_t)which) * kvq_tile_code_bytes(b);
                const size_t tok_seg = (size_t)pg * P + tl - sg.token_begin;
                uint8_t* row = oc + ((size_t)u * n_seg + tok_seg) * row_bytes;
                std::memset(row, 0, row_bytes);
                for (int d = 0; d < KVQ_D; ++d) {
                    int lane, slot;
                    if (which == KVQ_WHICH_K) kvq_k_slot(t, d, &lane, &slot);
                    else kvq_v_slot(t, d, &lane, &slot);
                    const uint32_t bit = (uint32_t)slot * b;
                    if (planes) {  // high-byte plane, then low-byte plane, each laid out like an 8-bit tile
                        row[2 * d] = tile[512u * 8 + kvq_tile_byte(lane, (uint32_t)slot)];
                        row[2 * d + 1] = tile[kvq_tile_byte(lane, (uint32_t)slot)];
                    } else if (b == 16) {
                        const uint8_t* src = tile + kvq_tile_byte(lane, bit / 8);
                        row[2 * d] = src[0];
                        row[2 * d + 1] = src[1];
                    } else {
                        uint32_t v = (tile[kvq_tile_byte(lane, bit / 8)] >> (bit % 8)) & ((1u << b) - 1u);
                        row[(size_t)d * b / 8] |= (uint8_t)(v << ((d * b) % 8));
                    }
                }
                if (meta_out) {
                    const uint16_t* m = reinterpret_cast<const uint16_t*>(meta.data() + tslot * KVQ_META_TILE_BYTES);
                    // the device keeps one (S, Z) per run of 32 channels (a group of 64 or 128 channels repeats
                    // its pair); the canonical format has one per group
                    const int gspan = c->cfg.group / KVQ_G, ngrp = KVQ_D / c->cfg.group;
                    for (int gg = 0; gg < ngrp; ++gg) {
                        const int g = gg * gspan;
                        size_t oi = ((size_t)u * n_seg + tok_seg) * ngrp + gg;
                        if (which == KVQ_WHICH_K) { os[oi] = m[t * 4 + g]; oz[oi] = m[128 + t * 4 + g]; }
                        else { os[oi] = m[256 + kvq_vmeta_index(t, g)]; oz[oi] = m[384 + kvq_vmeta_index(t, g)]; }
                    }
                }
            }
        }
    }
    return KVQ_OK;
}

kvq_status_t kvq_cache_set_option(kvq_cache_t* c, int32_t option, int32_t value) {
    if (!c) return KVQ_E_INVALID;
    switch (option) {
        case KVQ_OPT_SPLITS:
            if (value < 0 || value > KVQ_MAX_SPLITS) return KVQ_E_INVALID;
            c->splits_override = value;
            return KVQ_OK;
        case KVQ_OPT_FUSED_MERGE:
            c->fused_merge = value ? 1 : 0;
            return KVQ_OK;
        case KVQ_OPT_DETERMINISTIC:
            c->deterministic = value ? 1 : 0;
            return KVQ_OK;
        case KVQ_OPT_SHIFT_STRATEGY:
            if (value != KVQ_SHIFT_EQUIVALENT && value != KVQ_SHIFT_DIRECT && value != KVQ_SHIFT_MODIFIED) return KVQ_E_INVALID;
            c->shift_strategy = value;
            return KVQ_OK;
        case KVQ_OPT_TIER16:
            if (value != KVQ_TIER16_FP16 && value != KVQ_TIER16_INT16) return KVQ_E_INVALID;
            for (const auto& L : c->layers)
                if (L.T != 0) return KVQ_E_STATE;  // the tier decides what every 16-bit page holds
            c->tier16 = value;
            return KVQ_OK;
        case KVQ_OPT_TILE_COST_2BIT:
        case KVQ_OPT_TILE_COST_4BIT:
        case KVQ_OPT_TILE_COST_8BIT:
        case KVQ_OPT_TILE_COST_16BIT:
            if (value < 1 || value > 1000000) return KVQ_E_INVALID;
            c->tile_cost[option - KVQ_OPT_TILE_COST_2BIT] = value;
            for (auto& L : c->layers) L.plan_tiles = -1;
            return KVQ_OK;
        default: return KVQ_E_INVALID;
    }
}

kvq_status_t kvq_cache_set_reparam(kvq_cache_t* c, int32_t layer, const float* lambda_dev, void* hip_stream) {
    if (!c || layer < 0 || layer >= c->cfg.n_layers) return KVQ_E_INVALID;
    Layer& L = c->layers[(size_t)layer];
    if (L.T != 0) return KVQ_E_STATE;
    if (!lambda_dev) { L.reparam = false; return KVQ_OK; }
    if (!c->dry) {
        kvq_status_t st = ensure_device(c, as_stream(hip_stream));
        if (st != KVQ_OK) return st;
        if (kvq_launch_reparam_store(lambda_dev, c->lambda_dev(layer), c->cfg.n_kv_heads * KVQ_D, as_stream(hip_stream)) != hipSuccess)
            return KVQ_E_HIP;
    }
    L.reparam = true;
    return KVQ_OK;
}

kvq_status_t kvq_calibrate_lambda(const void* k_calib_dev, int32_t batch, int32_t n_kv_heads, int32_t n_tokens,
                                  float alpha, float* lambda_dev, void* hip_stream) {
    if (!k_calib_dev || !lambda_dev || batch < 1 || n_kv_heads < 1 || n_tokens < 1 || !(alpha >= 0.0f && alpha <= 4.0f))
        return KVQ_E_INVALID;
    return kvq_launch_calibrate(k_calib_dev, batch, n_kv_heads, n_tokens, alpha, 1.0e-5f, lambda_dev,
                                as_stream(hip_stream)) == hipSuccess ? KVQ_OK : KVQ_E_HIP;
}

namespace {
kvq_status_t cache_error(kvq_cache_t* c, int32_t layer, bool l1, const void* k_ref_dev, const void* v_ref_dev,
                         const float* gk_dev, const float* gv_dev, double* out_host, void* hip_stream) {
    if (!c || layer < 0 || layer >= c->cfg.n_layers || !k_ref_dev || !v_ref_dev || !out_host) return KVQ_E_INVALID;
    if (c->dry) return KVQ_E_STATE;
    const Layer& L = c->layers[(size_t)layer];
    if (L.T == 0) return KVQ_E_STATE;
    hipStream_t s = as_stream(hip_stream);
    double* err = reinterpret_cast<double*>(c->arena + c->flags_off + 16);  // two accumulators behind the flags
    if (kvq_launch_fill_u32(reinterpret_cast<uint32_t*>(err), 0u, 4, s) != hipSuccess) return KVQ_E_HIP;
    if (kvq_launch_error(l1, c->arena, c->table_dev(layer), k_ref_dev, v_ref_dev, gk_dev, gv_dev, L.T, c->tpp, c->units,
                         err, s) != hipSuccess)
        return KVQ_E_HIP;
    if (hipMemcpyAsync(out_host, err, 2 * sizeof(double), hipMemcpyDeviceToHost, s) != hipSuccess) return KVQ_E_HIP;
    if (hipStreamSynchronize(s) != hipSuccess) return KVQ_E_HIP;
    return KVQ_OK;
}
}  // namespace

kvq_status_t kvq_cache_sq_error(kvq_cache_t* c, int32_t layer, const void* k_ref_dev, const void* v_ref_dev,
                                double* sq_err_host, void* hip_stream) {
    return cache_error(c, layer, false, k_ref_dev, v_ref_dev, nullptr, nullptr, sq_err_host, hip_stream);
}

kvq_status_t kvq_cache_sensitivity(kvq_cache_t* c, int32_t layer, const void* k_ref_dev, const void* v_ref_dev,
                                   const float* gk_dev, const float* gv_dev, double* s_host, void* hip_stream) {
    return cache_error(c, layer, true, k_ref_dev, v_ref_dev, gk_dev, gv_dev, s_host, hip_stream);
}

// Eq. 6 of Sec. 3.2, exactly: multiple-choice knapsack by the list of non-dominated (memory, cost) states
// (Nemhauser-Ullmann).  After block i the list holds, by increasing memory and strictly decreasing cost, every
// total that no other choice of widths for blocks 0..i beats in both; a state remembers its predecessor and choice.
kvq_status_t kvq_allocate_bits(int32_t n_blocks, int32_t n_choices, const double* s, const uint64_t* mem,
                               uint64_t budget, int32_t* choice_out, double* total_s_out, uint64_t* total_mem_out) {
    if (n_blocks < 1 || n_blocks > 4096 || n_choices < 1 || n_choices > 16 || !s || !mem || !choice_out) return KVQ_E_INVALID;
    for (int64_t i = 0; i < (int64_t)n_blocks * n_choices; ++i)
        if (!(s[i] >= 0.0) || !std::isfinite(s[i])) return KVQ_E_INVALID;
    struct State { uint64_t m; double cost; int32_t prev; int32_t choice; };
    const size_t kMaxStates = 1u << 22;
    std::vector<std::vector<State>> layers((size_t)n_blocks);
    std::vector<State> cur{State{0, 0.0, -1, -1}}, cand;
    for (int i = 0; i < n_blocks; ++i) {
        cand.clear();
        for (int32_t p = 0; p < (int32_t)cur.size(); ++p)
            for (int32_t ch = 0; ch < n_choices; ++ch) {
                const uint64_t m = cur[(size_t)p].m + mem[(size_t)i * n_choices + ch];
                if (m < cur[(size_t)p].m || m > budget) continue;  // overflow or over budget
                cand.push_back(State{m, cur[(size_t)p].cost + s[(size_t)i * n_choices + ch], p, ch});
            }
        if (cand.empty()) return KVQ_E_BUDGET;
        // by memory, then cost, then (for reproducible ties) predecessor and choice
        std::sort(cand.begin(), cand.end(), [](const State& a, const State& b) {
            if (a.m != b.m) return a.m < b.m;
            if (a.cost != b.cost) return a.cost < b.cost;
            if (a.prev != b.prev) return a.prev < b.prev;
            return a.choice < b.choice;
        });
        std::vector<State>& keep = layers[(size_t)i];
        double best = std::numeric_limits<double>::infinity();
        for (const State& st : cand)
            if (st.cost < best) { keep.push_back(st); best = st.cost; }
        if (keep.size() > kMaxStates) return KVQ_E_OOM;
        cur = keep;
    }
    // the cheapest state is the last one (largest memory within the budget)
    int32_t at = (int32_t)layers[(size_t)n_blocks - 1].size() - 1;
    const State fin = layers[(size_t)n_blocks - 1][(size_t)at];
    for (int i = n_blocks - 1; i >= 0; --i) {
        const State& st = layers[(size_t)i][(size_t)at];
        choice_out[i] = st.choice;
        at = st.prev;
    }
    if (total_s_out) *total_s_out = fin.cost;
    if (total_mem_out) *total_mem_out = fin.m;
    return KVQ_OK;
}

kvq_status_t kvq_stream_read_probe(kvq_cache_t* c, const void* buf_dev, uint64_t bytes, int32_t n_workgroups,
                                   void* hip_stream) {
    if (!c || c->dry || !buf_dev || bytes < 16 || n_workgroups < 1 || n_workgroups > (1 << 20)) return KVQ_E_INVALID;
    if (reinterpret_cast<uintptr_t>(buf_dev) & 15u) return KVQ_E_INVALID;
    uint32_t* sink = reinterpret_cast<uint32_t*>(c->arena + c->jobs_off);  // never written in practice
    return kvq_launch_stream_read(buf_dev, bytes, n_workgroups, sink, as_stream(hip_stream)) == hipSuccess ? KVQ_OK : KVQ_E_HIP;
}

kvq_status_t kvq_cache_reset(kvq_cache_t* c, int32_t layer) {
    if (!c || layer < -1 || layer >= c->cfg.n_layers) return KVQ_E_INVALID;
    const int first = layer < 0 ? 0 : layer, last = layer < 0 ? c->cfg.n_layers : layer + 1;
    for (int l = first; l < last; ++l) {
        Layer& L = c->layers[(size_t)l];
        for (const Page& p : L.pages) {
            c->buddy.release(p.code_unit, order_of_bits(p.bits));
            if (c->has_meta(p.bits)) c->buddy.release(p.meta_unit, 0);
        }
        L.pages.clear();
        L.T = 0;
        L.version++;
        L.plan_tiles = -1;
        L.poisoned = false;
    }
    // An empty cache starts over: the next enqueueing call clears the device flags again (in stream order), among them
    // the mark that some V scale was large, which would otherwise outlive the data that set it.
    bool all_empty = true;
    for (const Layer& L : c->layers) all_empty = all_empty && L.T == 0;
    if (all_empty) c->device_ready = false;
    return KVQ_OK;
}

uint64_t kvq_cache_arena_free_bytes(const kvq_cache_t* c) { return c ? c->buddy.free_units() * c->unit_bytes : 0; }

const char* kvq_status_string(kvq_status_t s) {
    switch (s) {
        case KVQ_OK: return "ok";
        case KVQ_E_INVALID: return "invalid argument or unsupported configuration";
        case KVQ_E_BUDGET: return "block byte budget exceeded or nothing left to shrink";
        case KVQ_E_OOM: return "arena out of memory";
        case KVQ_E_STATE: return "call does not fit the cache state";
        case KVQ_E_HIP: return "HIP runtime error";
        case KVQ_E_LIMIT: return "launch exceeds the static scratch of kvq_decode_attention_static";
    }
    return "unknown status";
}

}  // extern "C"
