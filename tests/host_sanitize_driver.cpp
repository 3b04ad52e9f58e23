// Exercises the host side of libtkv (allocators, page tables, planners, residual routing, tagger, bit allocation)
// under AddressSanitizer / UndefinedBehaviorSanitizer.  Built and run by tests/test_host_sanitizers.py with the
// host compiler only; the kernel launchers are stubbed out (nothing here needs a GPU).
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <vector>

#include "tkv.h"
#include "tkv_internal.h"

int tkv_launch_append(const tkv_desc *, void *, uint8_t *, const void *, const void *, const uint8_t *, int32_t,
                      const int32_t *, const int32_t *, int32_t, int32_t *, void *) { return TKV_OK; }
int tkv_launch_gather(const tkv_desc *, const void *, const uint8_t *, const int32_t *, const int32_t *, int32_t, void *,
                      void *, int32_t, int32_t *, void *) { return TKV_OK; }
int tkv_launch_probe_read(const void *, size_t, uint32_t *, void *) { return TKV_OK; }
int tkv_launch_probe_records(const tkv_desc *, const void *, const int32_t *, const int32_t *, const int32_t *, const int32_t *,
                             const int32_t *, int32_t, int32_t, int32_t, uint32_t *, void *) { return TKV_OK; }
int tkv_launch_probe_mix(const void *, void *, size_t, int32_t, int32_t, void *) { return TKV_OK; }
int tkv_launch_decode_split(const tkv_desc *, const void *, const uint8_t *, const void *, const int32_t *, const int32_t *,
                            const int32_t *, const int32_t *, const int32_t *, int32_t, int32_t, int32_t, float, void *,
                            int32_t *, void *) { return TKV_OK; }
int tkv_launch_decode_reduce(const tkv_desc *, const int32_t *, int32_t, int32_t, int32_t, float *, const void *, void *) { return TKV_OK; }

#define CHECK(x) do { if (!(x)) { std::printf("FAILED line %d: %s\n", __LINE__, #x); return 1; } } while (0)

static uint64_t rng_state = 88172645463325252ull;
static uint32_t rnd() { rng_state ^= rng_state << 13; rng_state ^= rng_state >> 7; rng_state ^= rng_state << 17; return (uint32_t)(rng_state >> 32); }

int main()
{
    for (int axis = 0; axis < 2; ++axis) {
        tkv_desc d = {4, 128, 32, 64, 40, 40, axis};
        tkv_alloc *a = nullptr;
        CHECK(tkv_alloc_create(&d, 7, &a) == TKV_OK);
        std::vector<tkv_seq *> seqs(5, nullptr);
        for (auto &s : seqs) CHECK(tkv_seq_create(&s) == TKV_OK);
        int32_t base = 0;
        for (int round = 0; round < 6; ++round)
            for (size_t b = 0; b < seqs.size(); ++b) {
                const int32_t n = (int32_t)(rnd() % 150);
                std::vector<uint8_t> tags((size_t)n), bits((size_t)n);
                for (auto &t : tags) t = (rnd() % 3) ? 2 : 4;
                CHECK(tkv_route_residual(tags.data(), n, bits.data()) == TKV_OK);
                const uint8_t *use = axis ? bits.data() : tags.data();
                const int32_t cap = tkv_plan_append_max_work(n);
                std::vector<int32_t> slots((size_t)n), wp((size_t)cap), ws((size_t)cap * 64);
                int32_t nw = -1;
                const int st = tkv_plan_append(a, seqs[b], use, n, base, slots.data(), wp.data(), ws.data(), cap, &nw);
                CHECK(st == TKV_OK || st == TKV_ERR_POOL_EXHAUSTED);
                if (st == TKV_OK) { CHECK(nw >= 0 && nw <= cap); base += n; }
            }
        // page tables and the decode plan
        std::vector<int32_t> indptr(1, 0), ids, n2, n4;
        for (auto *s : seqs) {
            const int32_t np = tkv_seq_n_pages(s, 2) + tkv_seq_n_pages(s, 4);
            const size_t old = ids.size();
            ids.resize(old + (size_t)np);
            CHECK(tkv_seq_page_ids(s, ids.data() + old, np) == np);
            indptr.push_back((int32_t)ids.size());
            n2.push_back(tkv_seq_n_tokens(s, 2));
            n4.push_back(tkv_seq_n_tokens(s, 4));
        }
        for (int32_t target : {1, 3, 17, 400}) {
            const int32_t cap = tkv_plan_decode_capacity((int32_t)seqs.size(), target);
            std::vector<int32_t> items((size_t)cap * 4), sip(seqs.size() + 1);
            const int32_t ni = tkv_plan_decode(&d, (int32_t)seqs.size(), indptr.data(), n2.data(), n4.data(), target,
                                               items.data(), cap, sip.data());
            CHECK(ni >= 0 && ni <= cap && sip.back() == ni);
        }
        CHECK(tkv_decode_workspace_bytes(&d, 10, 8) > 0);
        for (auto *s : seqs) { CHECK(tkv_seq_release(s, a) == TKV_OK); tkv_seq_destroy(s); }
        CHECK(tkv_alloc_free_count(a, 2) == 40 && tkv_alloc_free_count(a, 4) == 40);
        tkv_alloc_destroy(a);
    }
    // tagger, counts, allocation, lookup
    {
        const int32_t n = 500;
        std::vector<uint8_t> sem((size_t)n), mod((size_t)n), tags((size_t)n), bits((size_t)n);
        for (int32_t t = 0; t < n; ++t) { sem[(size_t)t] = (uint8_t)(rnd() % 7); mod[(size_t)t] = (uint8_t)(sem[(size_t)t] == 5 ? rnd() % 2 : 0); }
        CHECK(tkv_tag_tokens(sem.data(), mod.data(), n, tags.data()) == TKV_OK);
        std::vector<int64_t> N(TKV_N_TAGS, 0);
        CHECK(tkv_tag_counts(tags.data(), n, N.data()) == TKV_OK);
        std::vector<double> D2(TKV_N_TAGS), D4(TKV_N_TAGS);
        for (int k = 0; k < TKV_N_TAGS; ++k) { D4[(size_t)k] = (rnd() % 100) * 0.01; D2[(size_t)k] = D4[(size_t)k] + (rnd() % 100) * 0.1; }
        std::vector<uint8_t> table(TKV_N_TAGS);
        CHECK(tkv_allocate_bits_greedy(TKV_N_TAGS, N.data(), D2.data(), D4.data(), 2.6, table.data()) == TKV_OK);
        CHECK(tkv_tags_to_bits(tags.data(), n, table.data(), bits.data()) == TKV_OK);
        std::vector<uint8_t> small(12);
        CHECK(tkv_allocate_bits_exhaustive(12, N.data(), D2.data(), D4.data(), 3.0, small.data()) == TKV_OK);
        CHECK(tkv_allocate_bits_exhaustive(23, N.data(), D2.data(), D4.data(), 3.0, table.data()) == TKV_ERR_INVALID_ARG);
    }
    std::printf("host sanitizer run ok\n");
    return 0;
}
