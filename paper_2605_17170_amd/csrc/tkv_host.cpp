// Host side of libtkv: geometry, the two page allocators, per-sequence page
// tables, the append and decode planners, the residual routing of per-channel
// INT2 keys, the triaxial tagger and the tag -> bitwidth allocation, and
// argument validation in front of the kernel launchers.  Nothing here touches
// the GPU; the launchers live in tkv_append.hip, tkv_gather.hip,
// tkv_decode.hip and tkv_probe.hip.
//
// Paper passages: offset-split shared address space and one allocator per
// pool, Sec. 3.2.2; per-token bitwidth array routing tokens to the pools and
// the INT2-first partition of the page table, Sec. 3.2.3; residual policy,
// Sec. 3.2.1; tag space, Sec. 3.1; budgeted allocation, Sec. 3.1.3.
#include "tkv.h"
#include "tkv_internal.h"

#include <algorithm>
#include <cmath>
#include <cstring>
#include <new>
#include <vector>

namespace {

constexpr int kHeadDim = 128, kGroup = 32, kPageTokens = 64;

bool desc_ok(const tkv_desc *d)
{
    return d && d->n_kv_heads > 0 && d->head_dim == kHeadDim && d->group_size == kGroup &&
           d->page_tokens == kPageTokens && d->n_pages_int2 >= 0 && d->n_pages_int4 >= 0 &&
           (int64_t)d->n_pages_int2 + d->n_pages_int4 <= INT32_MAX / kPageTokens &&
           (d->int2_key_axis == TKV_KEYS_PER_TOKEN || d->int2_key_axis == TKV_KEYS_PER_CHANNEL);
}

int desc_status(const tkv_desc *d)
{
    if (!d) return TKV_ERR_INVALID_ARG;
    return desc_ok(d) ? TKV_OK : TKV_ERR_BAD_SHAPE;
}

// splitmix64: seeds and drives the free-list shuffle
inline uint64_t mix64(uint64_t &s)
{
    uint64_t z = (s += 0x9E3779B97F4A7C15ull);
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}

inline int32_t ceil_div(int32_t a, int32_t b) { return (a + b - 1) / b; }

} // namespace

struct tkv_alloc {
    tkv_desc desc;
    std::vector<int32_t> free_list[2];   // [0] INT2 pool, [1] INT4 pool; back() is handed out next
    std::vector<uint8_t> in_use;         // per page
};

struct tkv_seq {
    std::vector<int32_t> pages[2];
    int32_t n_tok[2] = {0, 0};
};

extern "C" {

const char *tkv_strerror(int status)
{
    switch (status) {
    case TKV_OK: return "ok";
    case TKV_ERR_INVALID_ARG: return "invalid argument";
    case TKV_ERR_BAD_BITS: return "bitwidth is not 2 or 4";
    case TKV_ERR_BAD_SHAPE: return "unsupported shape";
    case TKV_ERR_PAGE_RANGE: return "page id out of range";
    case TKV_ERR_POOL_EXHAUSTED: return "pool exhausted";
    case TKV_ERR_WORKSPACE_TOO_SMALL: return "workspace too small";
    case TKV_ERR_HIP: return "HIP launch failed";
    case TKV_ERR_CAPACITY: return "output array too small";
    default: return "unknown status";
    }
}

size_t tkv_record_bytes(int bits)
{
    if (bits != 2 && bits != 4) return 0;
    const size_t codes = (size_t)kPageTokens * kHeadDim * bits / 8;
    const size_t meta = (size_t)kPageTokens * (kHeadDim / kGroup) * 2;   // fp16 per (token, group)
    return 2 * (codes + 2 * meta);
}

size_t tkv_page_bytes(const tkv_desc *desc, int bits)
{
    if (!desc_ok(desc)) return 0;
    return tkv_record_bytes(bits) * (size_t)desc->n_kv_heads;
}

size_t tkv_pool_bytes(const tkv_desc *desc)
{
    if (!desc_ok(desc)) return 0;
    return tkv_page_bytes(desc, 2) * (size_t)desc->n_pages_int2 +
           tkv_page_bytes(desc, 4) * (size_t)desc->n_pages_int4;
}

size_t tkv_record_offset(const tkv_desc *desc, int32_t page, int32_t head)
{
    if (!desc_ok(desc) || page < 0 || head < 0 || head >= desc->n_kv_heads ||
        page >= desc->n_pages_int2 + desc->n_pages_int4)
        return (size_t)-1;
    if (page < desc->n_pages_int2)
        return ((size_t)page * desc->n_kv_heads + head) * tkv_record_bytes(2);
    return tkv_page_bytes(desc, 2) * (size_t)desc->n_pages_int2 +
           ((size_t)(page - desc->n_pages_int2) * desc->n_kv_heads + head) * tkv_record_bytes(4);
}

/* ---------------------------------------------------------------- allocator */

int tkv_alloc_create(const tkv_desc *desc, uint64_t shuffle_seed, tkv_alloc **out)
{
    if (!out) return TKV_ERR_INVALID_ARG;
    *out = nullptr;
    if (int st = desc_status(desc)) return st;
    tkv_alloc *a = new (std::nothrow) tkv_alloc;
    if (!a) return TKV_ERR_INVALID_ARG;
    a->desc = *desc;
    const int32_t n[2] = {desc->n_pages_int2, desc->n_pages_int4};
    const int32_t base[2] = {0, desc->n_pages_int2};
    a->in_use.assign((size_t)n[0] + n[1], 0);
    uint64_t state = shuffle_seed;
    for (int p = 0; p < 2; ++p) {
        auto &fl = a->free_list[p];
        fl.resize((size_t)n[p]);
        // back() is handed out first: store in decreasing order so that
        // an unshuffled allocator returns increasing page ids
        for (int32_t i = 0; i < n[p]; ++i) fl[(size_t)i] = base[p] + n[p] - 1 - i;
        if (shuffle_seed)
            for (int32_t i = n[p] - 1; i > 0; --i)
                std::swap(fl[(size_t)i], fl[(size_t)(mix64(state) % (uint64_t)(i + 1))]);
    }
    *out = a;
    return TKV_OK;
}

void tkv_alloc_destroy(tkv_alloc *a) { delete a; }

int tkv_alloc_pages(tkv_alloc *a, int bits, int32_t n, int32_t *page_ids_out)
{
    if (!a || n < 0 || (n > 0 && !page_ids_out)) return TKV_ERR_INVALID_ARG;
    if (bits != 2 && bits != 4) return TKV_ERR_BAD_BITS;
    auto &fl = a->free_list[bits == 4];
    if ((size_t)n > fl.size()) return TKV_ERR_POOL_EXHAUSTED;
    for (int32_t i = 0; i < n; ++i) {
        page_ids_out[i] = fl.back();
        fl.pop_back();
        a->in_use[(size_t)page_ids_out[i]] = 1;
    }
    return TKV_OK;
}

int tkv_free_pages(tkv_alloc *a, const int32_t *page_ids, int32_t n)
{
    if (!a || n < 0 || (n > 0 && !page_ids)) return TKV_ERR_INVALID_ARG;
    const int32_t total = a->desc.n_pages_int2 + a->desc.n_pages_int4;
    // validate first (including duplicates inside the request), then free
    std::vector<int32_t> sorted(page_ids, page_ids + n);
    std::sort(sorted.begin(), sorted.end());
    for (int32_t i = 0; i < n; ++i) {
        const int32_t p = sorted[(size_t)i];
        if (p < 0 || p >= total || !a->in_use[(size_t)p]) return TKV_ERR_PAGE_RANGE;
        if (i && sorted[(size_t)i - 1] == p) return TKV_ERR_PAGE_RANGE;
    }
    for (int32_t i = 0; i < n; ++i) {
        const int32_t p = page_ids[i];
        a->in_use[(size_t)p] = 0;
        a->free_list[p >= a->desc.n_pages_int2].push_back(p);
    }
    return TKV_OK;
}

int32_t tkv_alloc_free_count(const tkv_alloc *a, int bits)
{
    if (!a) return TKV_ERR_INVALID_ARG;
    if (bits != 2 && bits != 4) return TKV_ERR_BAD_BITS;
    return (int32_t)a->free_list[bits == 4].size();
}

/* ---------------------------------------------------------------- sequences */

int tkv_seq_create(tkv_seq **out)
{
    if (!out) return TKV_ERR_INVALID_ARG;
    *out = new (std::nothrow) tkv_seq;
    return *out ? TKV_OK : TKV_ERR_INVALID_ARG;
}

void tkv_seq_destroy(tkv_seq *s) { delete s; }

int tkv_seq_release(tkv_seq *s, tkv_alloc *a)
{
    if (!s || !a) return TKV_ERR_INVALID_ARG;
    for (int p = 0; p < 2; ++p) {
        int st = tkv_free_pages(a, s->pages[p].data(), (int32_t)s->pages[p].size());
        if (st) return st;
        s->pages[p].clear();
        s->n_tok[p] = 0;
    }
    return TKV_OK;
}

int32_t tkv_seq_n_tokens(const tkv_seq *s, int bits)
{
    if (!s) return TKV_ERR_INVALID_ARG;
    if (bits != 2 && bits != 4) return TKV_ERR_BAD_BITS;
    return s->n_tok[bits == 4];
}

int32_t tkv_seq_n_pages(const tkv_seq *s, int bits)
{
    if (!s) return TKV_ERR_INVALID_ARG;
    if (bits != 2 && bits != 4) return TKV_ERR_BAD_BITS;
    return (int32_t)s->pages[bits == 4].size();
}

int32_t tkv_seq_page_ids(const tkv_seq *s, int32_t *out, int32_t capacity)
{
    if (!s || capacity < 0 || (capacity > 0 && !out)) return TKV_ERR_INVALID_ARG;
    const size_t n = s->pages[0].size() + s->pages[1].size();
    if (n > (size_t)capacity) return TKV_ERR_CAPACITY;
    if (!s->pages[0].empty()) std::memcpy(out, s->pages[0].data(), s->pages[0].size() * sizeof(int32_t));
    if (!s->pages[1].empty())
        std::memcpy(out + s->pages[0].size(), s->pages[1].data(), s->pages[1].size() * sizeof(int32_t));
    return (int32_t)n;
}

/* ---------------------------------------------------------------- Q1: append plan */

int tkv_route_residual(const uint8_t *tag_bits, int32_t n_tokens, uint8_t *bits_out)
{
    if (n_tokens < 0 || (n_tokens > 0 && (!tag_bits || !bits_out))) return TKV_ERR_INVALID_ARG;
    int32_t n2 = 0;
    for (int32_t t = 0; t < n_tokens; ++t) {
        if (tag_bits[t] != 2 && tag_bits[t] != 4) return TKV_ERR_BAD_BITS;
        n2 += tag_bits[t] == 2;
    }
    int32_t keep = n2 - n2 % kGroup;   // INT2 tokens that fill whole blocks, counted from the front
    for (int32_t t = 0; t < n_tokens; ++t) {
        uint8_t b = tag_bits[t];
        if (b == 2 && keep-- <= 0) b = 4;
        bits_out[t] = b;
    }
    return TKV_OK;
}

int32_t tkv_plan_append_max_work(int32_t n_tokens)
{
    if (n_tokens < 0) return TKV_ERR_INVALID_ARG;
    // each width touches at most one partly filled page plus ceil(n/64) new ones
    return n_tokens / kPageTokens + 4;
}

int tkv_plan_append(tkv_alloc *a, tkv_seq *s, const uint8_t *tag_bits, int32_t n_tokens,
                    int32_t token_base, int32_t *slot_ids_out, int32_t *work_pages_out,
                    int32_t *work_src_out, int32_t max_work, int32_t *n_work_out)
{
    if (!a || !s || n_tokens < 0 || token_base < 0 || max_work < 0 || !n_work_out) return TKV_ERR_INVALID_ARG;
    if (n_tokens > 0 && (!tag_bits || !slot_ids_out)) return TKV_ERR_INVALID_ARG;
    if (max_work > 0 && (!work_pages_out || !work_src_out)) return TKV_ERR_INVALID_ARG;
    if ((int64_t)token_base + n_tokens > INT32_MAX) return TKV_ERR_INVALID_ARG;
    *n_work_out = 0;
    int32_t n_new[2] = {0, 0};
    for (int32_t t = 0; t < n_tokens; ++t) {
        if (tag_bits[t] != 2 && tag_bits[t] != 4) return TKV_ERR_BAD_BITS;
        ++n_new[tag_bits[t] == 4];
    }
    if (a->desc.int2_key_axis == TKV_KEYS_PER_CHANNEL && n_new[0] % kGroup) return TKV_ERR_INVALID_ARG;
    int32_t room[2], new_pages[2], touched = 0;
    for (int p = 0; p < 2; ++p) {
        room[p] = (int32_t)s->pages[p].size() * kPageTokens - s->n_tok[p];   // free slots of the open page
        new_pages[p] = n_new[p] > room[p] ? ceil_div(n_new[p] - room[p], kPageTokens) : 0;
        if ((size_t)new_pages[p] > a->free_list[p].size()) return TKV_ERR_POOL_EXHAUSTED;
        touched += new_pages[p] + (n_new[p] > 0 && room[p] > 0);
    }
    if (touched > max_work) return TKV_ERR_CAPACITY;

    // commit: take pages, then lay the work list out as [INT2 pages..., INT4 pages...]
    int32_t first_work[2], first_page_index[2];
    int32_t w = 0;
    for (int p = 0; p < 2; ++p) {
        const bool open = n_new[p] > 0 && room[p] > 0;
        first_page_index[p] = (int32_t)s->pages[p].size() - (open ? 1 : 0);   // index in the stream of the first touched page
        const size_t old = s->pages[p].size();
        s->pages[p].resize(old + (size_t)new_pages[p]);
        tkv_alloc_pages(a, p ? 4 : 2, new_pages[p], s->pages[p].data() + old);   // cannot fail: checked above
        first_work[p] = w;
        if (n_new[p] == 0) continue;
        for (size_t i = (size_t)first_page_index[p]; i < s->pages[p].size(); ++i) work_pages_out[w++] = s->pages[p][i];
    }
    std::fill(work_src_out, work_src_out + (size_t)w * kPageTokens, -1);
    int32_t cursor[2] = {s->n_tok[0], s->n_tok[1]};   // position in the stream of the next token
    for (int32_t t = 0; t < n_tokens; ++t) {
        const int p = tag_bits[t] == 4;
        const int32_t pos = cursor[p]++;
        const int32_t page_index = pos / kPageTokens, slot = pos % kPageTokens;
        slot_ids_out[t] = s->pages[p][(size_t)page_index] * kPageTokens + slot;
        work_src_out[(size_t)(first_work[p] + page_index - first_page_index[p]) * kPageTokens + slot] = token_base + t;
    }
    s->n_tok[0] = cursor[0];
    s->n_tok[1] = cursor[1];
    *n_work_out = w;
    return TKV_OK;
}

/* ---------------------------------------------------------------- D1: decode plan */

int32_t tkv_plan_decode_capacity(int32_t batch, int32_t target_items)
{
    if (batch < 0 || target_items < 1 || (int64_t)batch + target_items > INT32_MAX) return TKV_ERR_INVALID_ARG;
    return batch + target_items;
}

int32_t tkv_plan_decode(const tkv_desc *desc, int32_t batch, const int32_t *page_indptr,
                        const int32_t *n_tok_int2, const int32_t *n_tok_int4,
                        int32_t target_items, int32_t *items_out, int32_t capacity,
                        int32_t *seq_item_indptr_out)
{
    if (int st = desc_status(desc)) return st;
    if (batch < 0 || target_items < 1 || capacity < 0 || !page_indptr || !seq_item_indptr_out) return TKV_ERR_INVALID_ARG;
    if (batch > 0 && (!n_tok_int2 || !n_tok_int4)) return TKV_ERR_INVALID_ARG;
    if (capacity > 0 && !items_out) return TKV_ERR_INVALID_ARG;
    // decode cost of a page: the kernel is bound by instruction issue, not bytes, and an INT4 page costs
    // about 7/6 of an INT2 page (same MFMA count, a few more unpack operations, more bytes in flight)
    constexpr int64_t kCost2 = 6, kCost4 = 7;
    int64_t total = 0;
    for (int32_t b = 0; b < batch; ++b) {
        if (n_tok_int2[b] < 0 || n_tok_int4[b] < 0) return TKV_ERR_INVALID_ARG;
        if (desc->int2_key_axis == TKV_KEYS_PER_CHANNEL && n_tok_int2[b] % kGroup) return TKV_ERR_INVALID_ARG;
        const int32_t p2 = ceil_div(n_tok_int2[b], kPageTokens), p4 = ceil_div(n_tok_int4[b], kPageTokens);
        if (page_indptr[b + 1] - page_indptr[b] != p2 + p4) return TKV_ERR_INVALID_ARG;
        total += kCost2 * p2 + kCost4 * p4;
    }
    // The launch ends with its slowest wavefront: find the smallest bound on an item's cost for which the batch
    // still splits into at most target_items items (every sequence into ceil(cost / bound) equal parts), so that no
    // item is heavier than the others by more than the rounding to whole pages.
    auto items_for = [&](int64_t bound) {
        int64_t n = 0;
        for (int32_t b = 0; b < batch; ++b) {
            const int64_t p2 = ceil_div(n_tok_int2[b], kPageTokens), p4 = ceil_div(n_tok_int4[b], kPageTokens);
            const int64_t cost = kCost2 * p2 + kCost4 * p4;
            if (cost > 0) n += std::min<int64_t>(p2 + p4, (cost + bound - 1) / bound);
        }
        return n;
    };
    int64_t lo = 1, hi = std::max<int64_t>(1, total);   // items_for(hi) <= number of non-empty sequences
    while (lo < hi) {
        const int64_t mid = lo + (hi - lo) / 2;
        if (items_for(mid) <= (int64_t)target_items) hi = mid;
        else lo = mid + 1;
    }
    const int64_t per_item = lo;   // with more non-empty sequences than target_items: one item each
    int32_t n_items = 0;
    seq_item_indptr_out[0] = 0;
    for (int32_t b = 0; b < batch; ++b) {
        const int32_t p2 = ceil_div(n_tok_int2[b], kPageTokens), p4 = ceil_div(n_tok_int4[b], kPageTokens);
        const int32_t pages = p2 + p4;
        const int64_t cost = kCost2 * p2 + kCost4 * p4;
        if (pages > 0) {
            const int32_t n_split = (int32_t)std::min<int64_t>(pages, (cost + per_item - 1) / per_item);
            if (n_items + n_split > capacity) return TKV_ERR_CAPACITY;
            int32_t begin = 0;
            int64_t cum = 0;   // cost of pages [0, begin)
            for (int32_t k = 0; k < n_split; ++k) {
                const int64_t goal = cost * (k + 1) / n_split;
                int32_t end = begin;
                while (end < pages && (end == begin || cum + (end < p2 ? kCost2 : kCost4) <= goal)) {
                    cum += end < p2 ? kCost2 : kCost4;
                    ++end;
                }
                end = std::min(end, pages - (n_split - 1 - k));   // leave a page for every later item
                if (k == n_split - 1) end = pages;
                // recompute cum if the clamp moved `end` backwards
                cum = kCost2 * std::min(end, p2) + kCost4 * std::max(0, end - p2);
                int32_t *it = items_out + 4 * (size_t)n_items;
                it[0] = b; it[1] = begin; it[2] = end; it[3] = n_items++;   // partial slot = place in sequence order
                begin = end;
            }
        }
        seq_item_indptr_out[b + 1] = n_items;
    }
    // Launch order.  The kernel runs one wavefront per (item, kv head), all resident at once, three to a SIMD, and the
    // hardware deals workgroups out in order: the items at places p, p + S and p + 2S of the list, S = target_items / 3,
    // share SIMDs.  A wavefront over INT2 pages keeps its SIMD busier than one over INT4 pages (same arithmetic, 40 %
    // fewer bytes to wait for), and three of them together run 3-12 % slower than in mixed company, which is what the
    // launch then ends with.  Listing the items by falling share of INT2 pages puts the INT2-heaviest third at the
    // places [0, S), the INT4-heaviest at [2S, 3S), one of each on every SIMD.  (Any order is correct: an item names
    // its own partial slot.)
    if (n_items > 1) {
        std::vector<int32_t> order(n_items);
        std::vector<int64_t> key(n_items);
        for (int32_t k = 0; k < n_items; ++k) {
            const int32_t *it = items_out + 4 * (size_t)k;
            const int64_t p2 = ceil_div(n_tok_int2[it[0]], kPageTokens);
            const int64_t a2 = std::max<int64_t>(0, std::min<int64_t>(it[2], p2) - it[1]), all = it[2] - it[1];
            order[k] = k;
            key[k] = all > 0 ? a2 * 4096 / all : 0;
        }
        std::stable_sort(order.begin(), order.end(), [&](int32_t x, int32_t y) { return key[x] > key[y]; });
        std::vector<int32_t> sorted(4 * (size_t)n_items);
        for (int32_t k = 0; k < n_items; ++k) std::copy_n(items_out + 4 * (size_t)order[k], 4, sorted.begin() + 4 * (size_t)k);
        std::copy(sorted.begin(), sorted.end(), items_out);
    }
    return n_items;
}

/* ---------------------------------------------------------------- device entry points */

int tkv_quantize_append(const tkv_desc *desc, void *pool, uint8_t *bit_map,
                        const void *K, const void *V, const uint8_t *tag_bits,
                        int32_t n_tokens, int32_t group_size,
                        const int32_t *work_pages, const int32_t *work_src, int32_t n_work,
                        int32_t *status, void *stream)
{
    if (int st = desc_status(desc)) return st;
    if (group_size != kGroup) return TKV_ERR_BAD_SHAPE;
    if (n_tokens < 0 || n_work < 0) return TKV_ERR_INVALID_ARG;
    if (n_work == 0) return TKV_OK;
    if (!pool || !bit_map || !K || !V || !tag_bits || !work_pages || !work_src) return TKV_ERR_INVALID_ARG;
    if (((uintptr_t)pool & 255) || ((uintptr_t)K & 15) || ((uintptr_t)V & 15)) return TKV_ERR_INVALID_ARG;
    if ((int64_t)n_work * desc->n_kv_heads > INT32_MAX) return TKV_ERR_INVALID_ARG;
    return tkv_launch_append(desc, pool, bit_map, K, V, tag_bits, n_tokens, work_pages, work_src, n_work, status, stream);
}

/* ---------------------------------------------------------------- T1: tagger */

int tkv_tag_tokens(const uint8_t *semantic, const uint8_t *modal, int32_t n_tokens, uint8_t *tags_out)
{
    if (n_tokens < 0 || (n_tokens > 0 && (!semantic || !modal || !tags_out))) return TKV_ERR_INVALID_ARG;
    constexpr uint8_t kUser = 1;
    for (int32_t t = 0; t < n_tokens; ++t)
        if (semantic[t] > 6 || modal[t] > 1) return TKV_ERR_INVALID_ARG;
    // one scan from the end: the number of user messages that start after a token is its distance in turns
    int32_t later = 0;
    for (int32_t t = n_tokens - 1; t >= 0; --t) {
        const int temporal = later > 2 ? 0 : 3 - later;
        tags_out[t] = (uint8_t)((temporal * 2 + modal[t]) * 7 + semantic[t]);
        later += semantic[t] == kUser && (t == 0 || semantic[t - 1] != kUser);
    }
    return TKV_OK;
}

int tkv_tags_to_bits(const uint8_t *tags, int32_t n_tokens, const uint8_t *table, uint8_t *bits_out)
{
    if (n_tokens < 0 || !table || (n_tokens > 0 && (!tags || !bits_out))) return TKV_ERR_INVALID_ARG;
    for (int k = 0; k < TKV_N_TAGS; ++k)
        if (table[k] != 2 && table[k] != 4) return TKV_ERR_BAD_BITS;
    for (int32_t t = 0; t < n_tokens; ++t)
        if (tags[t] >= TKV_N_TAGS) return TKV_ERR_INVALID_ARG;
    for (int32_t t = 0; t < n_tokens; ++t) bits_out[t] = table[tags[t]];
    return TKV_OK;
}

int tkv_tag_counts(const uint8_t *tags, int32_t n_tokens, int64_t *counts)
{
    if (n_tokens < 0 || !counts || (n_tokens > 0 && !tags)) return TKV_ERR_INVALID_ARG;
    for (int32_t t = 0; t < n_tokens; ++t)
        if (tags[t] >= TKV_N_TAGS) return TKV_ERR_INVALID_ARG;
    for (int32_t t = 0; t < n_tokens; ++t) ++counts[tags[t]];
    return TKV_OK;
}

int tkv_probe_stream_read(const void *buf, size_t bytes, uint32_t *sink, void *stream)
{
    if (bytes == 0) return TKV_OK;
    if (!buf || ((uintptr_t)buf & 15) || (bytes & 15)) return TKV_ERR_INVALID_ARG;
    return tkv_launch_probe_read(buf, bytes, sink, stream);
}

int tkv_probe_decode_reads(const tkv_desc *desc, const void *pool, const int32_t *page_indptr, const int32_t *page_ids,
                           const int32_t *n_tok_int2, const int32_t *n_tok_int4, const int32_t *items, int32_t n_items,
                           int32_t batch, int32_t walk, uint32_t *sink, void *stream)
{
    if (int st = desc_status(desc)) return st;
    if (n_items < 0 || batch < 0 || (walk != 0 && walk != 1)) return TKV_ERR_INVALID_ARG;
    if ((int64_t)n_items * desc->n_kv_heads > INT32_MAX) return TKV_ERR_INVALID_ARG;
    if (n_items == 0 || desc->n_pages_int2 + desc->n_pages_int4 == 0) return TKV_OK;
    if (!pool || ((uintptr_t)pool & 255)) return TKV_ERR_INVALID_ARG;
    if (walk && (batch == 0 || !page_indptr || !page_ids || !n_tok_int2 || !n_tok_int4 || !items)) return TKV_ERR_INVALID_ARG;
    return tkv_launch_probe_records(desc, pool, page_indptr, page_ids, n_tok_int2, n_tok_int4, items, n_items, batch, walk,
                                    sink, stream);
}

int tkv_probe_stream_mix(const void *src, void *dst, size_t unit_bytes, int32_t read_parts, int32_t write_parts, void *stream)
{
    const bool known = (read_parts == 4 && write_parts == 1) || (read_parts == 1 && write_parts == 4) ||
                       (read_parts == 1 && write_parts == 1);
    if (!known || (unit_bytes & 15)) return TKV_ERR_INVALID_ARG;
    if (unit_bytes == 0) return TKV_OK;
    if (!src || !dst || ((uintptr_t)src & 15) || ((uintptr_t)dst & 15)) return TKV_ERR_INVALID_ARG;
    return tkv_launch_probe_mix(src, dst, unit_bytes / 16, read_parts, write_parts, stream);
}

namespace {
int alloc_args_status(int32_t n_tags, const int64_t *N, const double *D2, const double *D4, double B, const uint8_t *out)
{
    if (n_tags < 0 || !(B >= 2.0) || !(B <= 4.0)) return TKV_ERR_INVALID_ARG;
    if (n_tags == 0) return TKV_OK;
    if (!N || !D2 || !D4 || !out) return TKV_ERR_INVALID_ARG;
    for (int32_t k = 0; k < n_tags; ++k)
        if (N[k] < 0 || !std::isfinite(D2[k]) || !std::isfinite(D4[k])) return TKV_ERR_INVALID_ARG;
    return TKV_OK;
}
// Largest admissible number of cache bits: B * sum N with a relative slack of 2^-40.
double alloc_limit(int32_t n_tags, const int64_t *N, double B, int64_t *sum_out)
{
    int64_t sum = 0;
    for (int32_t k = 0; k < n_tags; ++k) sum += N[k];
    *sum_out = sum;
    const double t = B * (double)sum;
    return t * (1.0 + std::ldexp(1.0, -40));
}
} // namespace

int tkv_allocate_bits_greedy(int32_t n_tags, const int64_t *N, const double *D2, const double *D4,
                             double B, uint8_t *bits_out)
{
    if (int st = alloc_args_status(n_tags, N, D2, D4, B, bits_out)) return st;
    if (n_tags == 0) return TKV_OK;
    std::vector<double> rho((size_t)n_tags);
    for (int32_t k = 0; k < n_tags; ++k) {
        const double gain = D2[k] - D4[k];
        if (N[k] == 0) rho[(size_t)k] = gain > 0 ? INFINITY : (gain < 0 ? -INFINITY : 0.0);
        else rho[(size_t)k] = gain / (2.0 * (double)N[k]);
    }
    std::vector<int32_t> order((size_t)n_tags);
    for (int32_t k = 0; k < n_tags; ++k) order[(size_t)k] = k;
    std::stable_sort(order.begin(), order.end(), [&](int32_t a, int32_t b) { return rho[(size_t)a] > rho[(size_t)b]; });
    int64_t sum = 0;
    const double limit = alloc_limit(n_tags, N, B, &sum);
    int64_t used = 2 * sum;
    for (int32_t k = 0; k < n_tags; ++k) bits_out[k] = 2;
    for (int32_t k : order)
        if ((double)(used + 2 * N[k]) <= limit) {
            bits_out[k] = 4;
            used += 2 * N[k];
        }
    return TKV_OK;
}

int tkv_allocate_bits_exhaustive(int32_t n_tags, const int64_t *N, const double *D2, const double *D4,
                                 double B, uint8_t *bits_out)
{
    if (n_tags > 22) return TKV_ERR_INVALID_ARG;
    if (int st = alloc_args_status(n_tags, N, D2, D4, B, bits_out)) return st;
    if (n_tags == 0) return TKV_OK;
    int64_t sum = 0;
    const double limit = alloc_limit(n_tags, N, B, &sum);
    bool have = false;
    double best_cost = 0.0;
    int64_t best_used = 0;
    uint32_t best_mask = 0;
    for (uint32_t mask = 0; mask < (1u << n_tags); ++mask) {
        int64_t used = 2 * sum;
        for (int32_t k = 0; k < n_tags; ++k)
            if ((mask >> k) & 1u) used += 2 * N[k];
        if ((double)used > limit) continue;
        double cost = 0.0;   // summed in tag order
        for (int32_t k = 0; k < n_tags; ++k) cost = cost + (((mask >> k) & 1u) ? D4[k] : D2[k]);
        if (!have || cost < best_cost || (cost == best_cost && used < best_used)) {
            have = true;
            best_cost = cost;
            best_used = used;
            best_mask = mask;
        }
    }
    for (int32_t k = 0; k < n_tags; ++k) bits_out[k] = ((best_mask >> k) & 1u) ? 4 : 2;
    return TKV_OK;
}

int tkv_gather_dequant(const tkv_desc *desc, const void *pool, const uint8_t *bit_map,
                       const int32_t *work_pages, const int32_t *work_dst, int32_t n_work,
                       void *K_out, void *V_out, int32_t n_tokens, int32_t *status, void *stream)
{
    if (int st = desc_status(desc)) return st;
    if (n_tokens < 0 || n_work < 0) return TKV_ERR_INVALID_ARG;
    if (n_work == 0) return TKV_OK;
    if (!pool || !bit_map || !K_out || !V_out || !work_pages || !work_dst) return TKV_ERR_INVALID_ARG;
    if (((uintptr_t)pool & 255) || ((uintptr_t)K_out & 15) || ((uintptr_t)V_out & 15)) return TKV_ERR_INVALID_ARG;
    if ((int64_t)n_work * desc->n_kv_heads > INT32_MAX) return TKV_ERR_INVALID_ARG;
    return tkv_launch_gather(desc, pool, bit_map, work_pages, work_dst, n_work, K_out, V_out, n_tokens, status, stream);
}

size_t tkv_decode_workspace_bytes(const tkv_desc *desc, int32_t n_items, int32_t n_q_heads)
{
    if (!desc_ok(desc) || n_items < 0 || n_q_heads <= 0) return 0;
    return (size_t)n_items * (size_t)n_q_heads * (size_t)(desc->head_dim + 2) * sizeof(float);
}

} // extern "C"

// Checks shared by the decode entry points.
int tkv_decode_check_args(const tkv_desc *desc, int32_t n_items, int32_t batch, int32_t n_q_heads,
                          const void *workspace, size_t workspace_bytes)
{
    if (int st = desc_status(desc)) return st;
    if (batch < 0 || n_items < 0 || n_q_heads <= 0) return TKV_ERR_INVALID_ARG;
    if (n_q_heads % desc->n_kv_heads) return TKV_ERR_BAD_SHAPE;
    const int r = n_q_heads / desc->n_kv_heads;
    if (r != 1 && r != 2 && r != 4 && r != 8) return TKV_ERR_BAD_SHAPE;
    if (n_items > 0 && !workspace) return TKV_ERR_INVALID_ARG;
    if ((uintptr_t)workspace & 15) return TKV_ERR_INVALID_ARG;
    if (workspace_bytes < tkv_decode_workspace_bytes(desc, n_items, n_q_heads)) return TKV_ERR_WORKSPACE_TOO_SMALL;
    if ((int64_t)n_items * desc->n_kv_heads > INT32_MAX || (int64_t)batch * n_q_heads > INT32_MAX) return TKV_ERR_INVALID_ARG;
    return TKV_OK;
}

extern "C" {

int tkv_decode_split(const tkv_desc *desc, const void *pool, const uint8_t *bit_map,
                     const void *q, const int32_t *page_indptr, const int32_t *page_ids,
                     const int32_t *n_tok_int2, const int32_t *n_tok_int4,
                     const int32_t *items, int32_t n_items, int32_t batch, int32_t n_q_heads,
                     float sm_scale, void *workspace, size_t workspace_bytes, int32_t *status, void *stream)
{
    if (int st = tkv_decode_check_args(desc, n_items, batch, n_q_heads, workspace, workspace_bytes)) return st;
    if (batch == 0 || n_items == 0) return TKV_OK;
    if (!(sm_scale > 0.0f) || !(sm_scale < 3.0e38f)) return TKV_ERR_INVALID_ARG;
    if (!q || !page_indptr || !n_tok_int2 || !n_tok_int4 || !pool || !bit_map || !page_ids || !items) return TKV_ERR_INVALID_ARG;
    if (((uintptr_t)pool & 255) || ((uintptr_t)q & 15)) return TKV_ERR_INVALID_ARG;
    return tkv_launch_decode_split(desc, pool, bit_map, q, page_indptr, page_ids, n_tok_int2, n_tok_int4, items,
                                   n_items, batch, n_q_heads, sm_scale, workspace, status, stream);
}

int tkv_decode_reduce(const tkv_desc *desc, const int32_t *seq_item_indptr, int32_t n_items,
                      int32_t batch, int32_t n_q_heads, float *out, const void *workspace,
                      size_t workspace_bytes, void *stream)
{
    if (int st = tkv_decode_check_args(desc, n_items, batch, n_q_heads, workspace, workspace_bytes)) return st;
    if (batch == 0) return TKV_OK;
    if (!out || !seq_item_indptr || ((uintptr_t)out & 15)) return TKV_ERR_INVALID_ARG;
    return tkv_launch_decode_reduce(desc, seq_item_indptr, n_items, batch, n_q_heads, out, workspace, stream);
}

int tkv_decode_attention(const tkv_desc *desc, const void *pool, const uint8_t *bit_map,
                         const void *q, const int32_t *page_indptr, const int32_t *page_ids,
                         const int32_t *n_tok_int2, const int32_t *n_tok_int4,
                         const int32_t *items, const int32_t *seq_item_indptr, int32_t n_items,
                         int32_t batch, int32_t n_q_heads, float sm_scale, float *out,
                         void *workspace, size_t workspace_bytes, int32_t *status, void *stream)
{
    // validate everything both launches need before launching anything
    if (int st = tkv_decode_check_args(desc, n_items, batch, n_q_heads, workspace, workspace_bytes)) return st;
    if (batch == 0) return TKV_OK;
    if (!(sm_scale > 0.0f) || !(sm_scale < 3.0e38f)) return TKV_ERR_INVALID_ARG;
    if (!q || !out || !page_indptr || !n_tok_int2 || !n_tok_int4 || !seq_item_indptr) return TKV_ERR_INVALID_ARG;
    if (n_items > 0 && (!pool || !bit_map || !page_ids || !items)) return TKV_ERR_INVALID_ARG;
    if (((uintptr_t)pool & 255) || ((uintptr_t)q & 15) || ((uintptr_t)out & 15)) return TKV_ERR_INVALID_ARG;
    if (int st = tkv_launch_decode_split(desc, pool, bit_map, q, page_indptr, page_ids, n_tok_int2, n_tok_int4, items,
                                         n_items, batch, n_q_heads, sm_scale, workspace, status, stream))
        return st;
    return tkv_launch_decode_reduce(desc, seq_item_indptr, n_items, batch, n_q_heads, out, workspace, stream);
}

} // extern "C"
