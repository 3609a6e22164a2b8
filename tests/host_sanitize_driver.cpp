// Random walk over the host side of the library (metadata-only pools: block allocator, block tables,
// reference counts, eviction, fork, truncate, batched steps, the taking back of half-done calls),
// meant to be built with -fsanitize=address,undefined on the host pass and run by
// tests/test_host_sanitizers.py.  Checks a shadow model as it goes; exits non-zero on a mismatch
// (the sanitizers abort by themselves).
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <map>
#include <vector>

#include "../include/sk.h"

static uint64_t rng_state = 0x5EED0009ull;
static uint32_t rnd(uint32_t n) { rng_state = rng_state * 6364136223846793005ull + 1442695040888963407ull; return (uint32_t)(rng_state >> 33) % n; }

#define CHECK(c) do { if (!(c)) { std::fprintf(stderr, "check failed at line %d: %s\n", __LINE__, #c); std::exit(1); } } while (0)

struct Shadow { int64_t len = 0, frozen = 0; };

int main(int argc, char** argv)
{
    const int n_ops = argc > 1 ? std::atoi(argv[1]) : 20000;
    for (int block_tokens : {16, 64}) {
        sk_pool_desc d = {};
        d.dtype = SK_BF16; d.n_q_heads = 32; d.n_kv_heads = 8; d.head_dim = 128;
        d.block_tokens = block_tokens; d.max_sessions = 12; d.n_blocks = 300; d.max_batch_tokens = 2048;
        d.flags = SK_POOL_METADATA_ONLY;
        sk_pool* p = nullptr;
        CHECK(sk_pool_create(&d, &p) == SK_OK && p);
        std::map<int32_t, Shadow> live;
        for (int it = 0; it < n_ops; ++it) {
            const uint32_t op = rnd(100);
            if (live.empty() || op < 8) {
                int32_t id = -1;
                const int rc = sk_session_create(p, &id);
                if ((int)live.size() == d.max_sessions) CHECK(rc == SK_E_NOMEM);
                else { CHECK(rc == SK_OK && !live.count(id)); live[id] = Shadow(); }
                continue;
            }
            auto itr = live.begin();
            std::advance(itr, rnd((uint32_t)live.size()));
            const int32_t id = itr->first;
            Shadow& s = itr->second;
            int64_t free_before = 0, len_before = 0;
            CHECK(sk_pool_blocks_free(p, &free_before) == SK_OK);
            CHECK(sk_session_length(p, id, &len_before) == SK_OK && len_before == s.len);
            if (op < 45) {                                   // append, sometimes with a failure ordered
                const int32_t L = 1 + (int32_t)rnd(rnd(4) == 0 ? 1500 : 90);
                const bool fail = rnd(5) == 0;
                if (fail) CHECK(sk_pool_inject_failure(p, 1 + (int32_t)rnd(6), 1) == SK_OK);
                const int rc = sk_session_append(p, id, nullptr, nullptr, nullptr, L, nullptr, SK_F32, nullptr, nullptr);
                CHECK(sk_pool_inject_failure(p, 0, 0) == SK_OK);
                if (rc == SK_OK) s.len += L;
                else {
                    int64_t len_after = 0;
                    CHECK(sk_session_length(p, id, &len_after) == SK_OK && len_after == s.len);
                    if (rc == SK_E_NOMEM) { int64_t f = 0; sk_pool_blocks_free(p, &f); CHECK(f == free_before); }
                }
            } else if (op < 55) {                            // truncate
                const int64_t nl = s.len ? (int64_t)rnd((uint32_t)s.len + 1) : 0;
                CHECK(sk_session_truncate(p, id, nl) == SK_OK);
                s.len = nl; if (s.frozen > nl) s.frozen = nl;
            } else if (op < 62) {                            // freeze (only grows; refused once tokens were evicted behind it)
                const int64_t nf = s.frozen + (int64_t)rnd((uint32_t)(s.len - s.frozen) + 1);
                if (sk_session_freeze(p, id, nf) == SK_OK) s.frozen = nf;
            } else if (op < 75) {                            // evict
                const int64_t room = s.len - s.frozen;
                const int64_t n = room ? (int64_t)rnd((uint32_t)room + 1) : 0;
                const bool fail = rnd(6) == 0;
                if (fail) CHECK(sk_pool_inject_failure(p, 1 + (int32_t)rnd(2), 1) == SK_OK);
                const int rc = sk_session_evict_oldest(p, id, n, nullptr);
                CHECK(sk_pool_inject_failure(p, 0, 0) == SK_OK);
                if (rc == SK_OK) s.len -= n; else CHECK(rc == SK_E_HIP);
                CHECK(sk_session_evict_oldest(p, id, s.len - s.frozen + 1, nullptr) == SK_E_INVAL);
            } else if (op < 85) {                            // fork a prefix
                const int64_t np = s.len ? (int64_t)rnd((uint32_t)s.len + 1) : 0;
                int32_t nid = -1;
                const int rc = sk_session_fork(p, id, np, &nid, nullptr);
                if (rc == SK_OK) { CHECK(!live.count(nid)); Shadow t; t.len = np; t.frozen = s.frozen < np ? s.frozen : np; live[nid] = t; }
                else CHECK(rc == SK_E_NOMEM);
            } else if (op < 92) {                            // destroy
                CHECK(sk_session_destroy(p, id) == SK_OK);
                live.erase(id);
                CHECK(sk_session_destroy(p, id) == SK_E_BADSESSION);
            } else {                                         // a ragged step over several sessions
                std::vector<int32_t> ids, ops, cu(1, 0);
                for (auto& kv : live) {
                    if (rnd(2)) continue;
                    const int32_t o = (int32_t)rnd(3);
                    if (o == SK_OP_QUERY_A && kv.second.len == 0) continue;
                    ids.push_back(kv.first); ops.push_back(o); cu.push_back(cu.back() + 1 + (int32_t)rnd(200));
                }
                if (ids.empty()) continue;
                const bool fail = rnd(4) == 0;
                if (fail) CHECK(sk_pool_inject_failure(p, rnd(2) ? SK_SITE_PLAN : 1 + (int32_t)rnd(5), 1) == SK_OK);
                const int rc = sk_batch_step(p, (int32_t)ids.size(), ids.data(), ops.data(), cu.data(), nullptr, nullptr, nullptr,
                                             nullptr, SK_F32, nullptr, nullptr);
                CHECK(sk_pool_inject_failure(p, 0, 0) == SK_OK);
                if (rc == SK_OK)
                    for (size_t i = 0; i < ids.size(); ++i)
                        if (ops[i] == SK_OP_APPEND) live[ids[i]].len += cu[i + 1] - cu[i];
            }
            // invariants after every operation: lengths, table sizes, block conservation
            int64_t free_now = 0;
            CHECK(sk_pool_blocks_free(p, &free_now) == SK_OK);
            std::map<int32_t, int> holders;
            for (auto& kv : live) {
                int64_t len = 0, nb = 0; const int32_t* tbl = nullptr;
                CHECK(sk_session_length(p, kv.first, &len) == SK_OK && len == kv.second.len);
                CHECK(sk_session_block_table(p, kv.first, &tbl, &nb) == SK_OK);
                CHECK(nb >= (len + block_tokens - 1) / block_tokens && nb <= (len + block_tokens - 1) / block_tokens + 2);
                for (int64_t i = 0; i < nb; ++i) { CHECK(tbl[i] >= 0 && tbl[i] < d.n_blocks); holders[tbl[i]]++; }
            }
            CHECK((int64_t)holders.size() + free_now == d.n_blocks);
        }
        for (auto& kv : live) CHECK(sk_session_destroy(p, kv.first) == SK_OK);
        int64_t f = 0;
        CHECK(sk_pool_blocks_free(p, &f) == SK_OK && f == d.n_blocks);
        CHECK(sk_pool_destroy(p) == SK_OK);
    }
    std::printf("host walk ok\n");
    return 0;
}
