// Host-side logic of the library under AddressSanitizer and UndefinedBehaviorSanitizer: the blob packer and its
// read-back, the cache / staging / swap bookkeeping and the error paths, driven through the C ABI in contexts
// without a GPU.  Every buffer handed to the library is a heap block of exactly the size the interface asks for, so
// an access one byte outside it is caught; the bookkeeping is followed by a brute-force LRU model (the k distinct
// most recently touched experts, found by scanning the history backwards) and by conservation checks.
// Built and run by tests/test_sanitized_host_logic.py; prints "ok" and exits 0 when nothing was found.
#include <algorithm>
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <random>
#include <set>
#include <vector>

#include "../../include/moe_offload.h"

#define CHECK(cond)                                                                         \
    do {                                                                                    \
        if (!(cond)) {                                                                      \
            std::fprintf(stderr, "%s:%d: check failed: %s (last error: %s)\n", __FILE__, __LINE__, #cond, moe_last_error()); \
            std::exit(1);                                                                   \
        }                                                                                   \
    } while (0)

namespace {

struct Arena {                       // exactly `bytes` of 64-byte aligned heap
    void *p = nullptr;
    explicit Arena(size_t bytes) { p = std::aligned_alloc(64, (bytes + 63) / 64 * 64); CHECK(p); }
    ~Arena() { std::free(p); }
};

moe_ctx_t *host_ctx(int n_staging, int max_batch, int hidden, int ffn, int top_k, uint64_t blob)
{
    moe_ctx_config_t c{n_staging, max_batch, hidden, ffn, top_k, MOE_CTX_HOST_ONLY, blob};
    moe_ctx_t *ctx = nullptr;
    CHECK(moe_ctx_create(&c, nullptr, 0, nullptr, nullptr, &ctx) == MOE_OK && ctx);
    return ctx;
}

// ---- blobs: pack every matrix of every expert, read every element of sampled rows back ------------------------------

void pack_and_peek(int H, int F, int bits, int group, int scale_group, std::mt19937 &rng)
{
    const uint64_t blob = moe_expert_blob_bytes_2level(H, F, bits, group, scale_group);
    if (blob == 0) return;          // a combination the library refuses (e.g. 2-bit with runs of 2 groups)
    const int E = 2;
    moe_layer_config_t lc{H, F, E, 2, bits, group, 2, 0, 0.f, 0, 0, scale_group};
    CHECK(moe_layer_host_bytes(&lc) == blob * E);
    moe_ctx_t *ctx = host_ctx(2, 1, H, F, 2, blob);
    Arena host(blob * E);
    std::vector<float> gate((size_t)E * H, 0.f);
    moe_layer_t *lay = nullptr;
    CHECK(moe_layer_create(ctx, &lc, gate.data(), nullptr, nullptr, host.p, &lay) == MOE_OK);
    for (int e = 0; e < E; ++e)
        for (int m = 0; m < 3; ++m) {
            const int rows = m == 2 ? H : F, cols = m == 2 ? F : H, groups = cols / group;
            const int run = scale_group ? std::min(scale_group, groups) : 0, runs = run ? (groups + run - 1) / run : 0;
            std::vector<uint8_t> q((size_t)rows * cols), sc((size_t)rows * groups), zc((size_t)rows * groups);
            std::vector<uint16_t> s((size_t)rows * groups), z((size_t)rows * groups), quad((size_t)rows * std::max(1, runs) * 4);
            for (auto &v : q) v = rng() % (1u << bits);
            for (auto &v : s) v = rng() & 0x7bff;           // finite fp16 patterns
            for (auto &v : z) v = rng() & 0x7bff;
            for (auto &v : sc) v = rng() & 255;
            for (auto &v : zc) v = rng() & 255;
            for (auto &v : quad) v = rng() & 0x7bff;
            if (scale_group) CHECK(moe_layer_load_expert_2level(lay, e, m, q.data(), sc.data(), zc.data(), quad.data()) == MOE_OK);
            else CHECK(moe_layer_load_expert(lay, e, m, q.data(), s.data(), z.data()) == MOE_OK);
            const int sample[4] = {0, rows - 1, (int)(rng() % rows), (int)(rng() % rows)};
            for (int r : sample)
                for (int c = 0; c < cols; ++c) {
                    uint8_t code; uint16_t a, b;
                    CHECK(moe_layer_peek_weight(lay, e, m, r, c, &code, &a, &b) == MOE_OK);
                    CHECK(code == q[(size_t)r * cols + c]);
                    const size_t g = (size_t)r * groups + c / group;
                    if (scale_group) {
                        uint16_t got[4];
                        CHECK(a == sc[g] && b == zc[g]);
                        CHECK(moe_layer_peek_run_meta(lay, e, m, r, c, got) == MOE_OK);
                        CHECK(std::memcmp(got, &quad[((size_t)r * runs + (c / group) / run) * 4], 8) == 0);
                    } else {
                        CHECK(a == s[g] && b == z[g]);
                    }
                }
            // a code above the format's range is refused, and nothing is written past the rows
            q[(size_t)(rows - 1) * cols + cols - 1] = (uint8_t)(1u << bits);
            const int32_t rc = scale_group ? moe_layer_load_expert_2level(lay, e, m, q.data(), sc.data(), zc.data(), quad.data())
                                           : moe_layer_load_expert(lay, e, m, q.data(), s.data(), z.data());
            CHECK(rc == MOE_EINVAL);
        }
    CHECK(moe_layer_destroy(lay) == MOE_OK && moe_ctx_destroy(ctx) == MOE_OK);
}

// ---- bookkeeping: random routing through moe_layer_resolve, followed by a history-replay model ----------------------

struct Brute {                       // one layer: the order in which experts touched the cache
    std::vector<int> history;
    std::vector<int> resident(int k) const
    {
        std::vector<int> seen;
        for (auto it = history.rbegin(); it != history.rend() && (int)seen.size() < k; ++it)
            if (std::find(seen.begin(), seen.end(), *it) == seen.end()) seen.push_back(*it);
        return seen;
    }
};

void bookkeeping(unsigned seed)
{
    std::mt19937 rng(seed);
    auto pick = [&](int lo, int hi) { return lo + (int)(rng() % (unsigned)(hi - lo + 1)); };
    const int E = pick(2, 16), K = pick(1, std::min(4, E)), k = pick(K, E), m = pick(0, 4), b = pick(0, 6), L = pick(1, 4);
    const int B = (rng() % 3 == 0) ? pick(2, 40) : 1, T = 24;
    const bool swap = rng() % 4 == 0, warm = swap || rng() % 3 == 0, no_cache = !swap && rng() % 8 == 0;
    const uint64_t blob = moe_expert_blob_bytes(64, 64, 4, 64);
    moe_ctx_t *ctx = host_ctx(b, B, 64, 64, K, blob);
    moe_layer_config_t lc{64, 64, E, K, 4, 64, k, m, 0.f, warm ? 1 : 0, (swap ? MOE_LAYER_SWAP : 0) | (no_cache ? MOE_LAYER_NO_CACHE : 0), 0};
    std::vector<float> gate((size_t)E * 64, 0.f);
    std::vector<Arena *> arenas;
    std::vector<moe_layer_t *> lay(L, nullptr);
    std::vector<Brute> brute(L);
    for (int l = 0; l < L; ++l) {
        arenas.push_back(new Arena(moe_layer_host_bytes(&lc)));
        CHECK(moe_layer_create(ctx, &lc, gate.data(), nullptr, nullptr, arenas.back()->p, &lay[l]) == MOE_OK);
        if (warm) {                                  // a warm start needs the experts it places: load all of them
            std::vector<uint8_t> q(64 * 64, 0);
            std::vector<uint16_t> s(64, 0x3c00), z(64, 0);
            for (int e = 0; e < E; ++e)
                for (int mtx = 0; mtx < 3; ++mtx) CHECK(moe_layer_load_expert(lay[l], e, mtx, q.data(), s.data(), z.data()) == MOE_OK);
            for (int e = 0; e < k; ++e) brute[l].history.push_back(e);
        }
    }
    std::vector<moe_step_trace_t> tr(1);
    uint64_t needed_total = 0;
    for (int t = 0; t < T; ++t)
        for (int l = 0; l < L; ++l) {
            std::vector<int32_t> idx((size_t)B * K);
            std::set<int> need;
            for (int bb = 0; bb < B; ++bb) {
                std::vector<int> perm(E);
                for (int e = 0; e < E; ++e) perm[e] = e;
                std::shuffle(perm.begin(), perm.end(), rng);
                for (int j = 0; j < K; ++j) { idx[(size_t)bb * K + j] = perm[j]; need.insert(perm[j]); }
            }
            std::vector<double> score(E);
            for (auto &v : score) v = (double)(rng() % 5);          // many ties
            moe_layer_t *next = l + 1 < L ? lay[l + 1] : nullptr;
            const std::vector<int> before = no_cache ? std::vector<int>() : brute[l].resident(k);
            CHECK(moe_layer_resolve(lay[l], next, idx.data(), B, next ? score.data() : nullptr, &tr[0]) == MOE_OK);
            const moe_step_trace_t &r = tr[0];
            CHECK(r.n_access == (int)need.size() && r.batch == B && r.top_k == K);
            needed_total += need.size();
            // order of the accesses: experts resident before the step first, then the absent ones, each ascending
            std::vector<int> res, abs;
            for (int e : need) (std::find(before.begin(), before.end(), e) != before.end() ? res : abs).push_back(e);
            for (int i = 0; i < r.n_access; ++i) {
                const moe_access_t &a = r.access[i];
                const bool was = i < (int)res.size();
                CHECK(a.expert == (was ? res[i] : abs[i - res.size()]));
                CHECK(was ? a.status == MOE_HIT : (a.status == MOE_MISS || a.status == MOE_PREFETCH_HIT));
                CHECK(a.slot >= 0 && a.slot < k && a.victim != a.expert && a.victim < E);
                brute[l].history.push_back(a.expert);
            }
            // what the cache holds afterwards: the k distinct most recently touched experts, each once
            std::vector<int32_t> slot_e(k), staged(MOE_MAX_EXPERTS);
            std::vector<uint64_t> stamp(k);
            int32_t n_staged = -1;
            CHECK(moe_layer_cache_state(lay[l], slot_e.data(), stamp.data(), staged.data(), &n_staged) == MOE_OK);
            std::vector<int> want = brute[l].resident(k), got;
            for (int e : slot_e) if (e >= 0) got.push_back(e);
            if (no_cache) {          // residency is forgotten before every step: only this step's experts can be there
                for (int e : got) CHECK(need.count(e));
            } else {
                std::sort(want.begin(), want.end());
                std::sort(got.begin(), got.end());
                CHECK(want == got);
            }
            CHECK(n_staged == 0);                                    // this layer's unused guesses were dropped
            if (next) {
                CHECK(r.n_guess == std::min(m, E));
                for (int i = 0; i + 1 < r.n_guess; ++i) {            // most likely first, ties to the lower id
                    const int a = r.guess_expert[i], c2 = r.guess_expert[i + 1];
                    CHECK(score[a] > score[c2] || (score[a] == score[c2] && a < c2));
                }
                int32_t ns = 0;
                CHECK(moe_layer_cache_state(lay[l + 1], nullptr, nullptr, staged.data(), &ns) == MOE_OK);
                CHECK(ns <= b && ns <= r.n_guess);
            }
            if (swap) {              // every expert in exactly one place; the host buffers a permutation with one spare
                std::vector<int32_t> hb(E);
                int32_t spare = -2;
                CHECK(moe_layer_placement(lay[l], hb.data(), &spare) == MOE_OK);
                std::set<int> used;
                int on_dev = 0;
                for (int e = 0; e < E; ++e) {
                    if (hb[e] < 0) { ++on_dev; CHECK(std::find(slot_e.begin(), slot_e.end(), e) != slot_e.end()); }
                    else { CHECK(hb[e] <= E - k && used.insert(hb[e]).second); }
                }
                CHECK(on_dev == k && spare >= 0 && spare <= E - k && !used.count(spare));
            }
        }
    uint64_t sum_needed = 0;
    for (int l = 0; l < L; ++l) {
        moe_stats_t st;
        CHECK(moe_layer_stats(lay[l], &st) == MOE_OK);
        CHECK(st.hits + st.prefetch_hits + st.misses == st.needed && st.steps == (uint64_t)T);
        CHECK(st.spec_issued >= st.prefetch_hits + st.spec_wasted);
        sum_needed += st.needed;
        // loading is over once a layer has stepped
        std::vector<uint8_t> q(64 * 64, 0);
        std::vector<uint16_t> s(64, 0x3c00), z(64, 0);
        CHECK(moe_layer_load_expert(lay[l], 0, 0, q.data(), s.data(), z.data()) == MOE_ESTATE);
    }
    CHECK(sum_needed == needed_total);
    for (int l = 0; l < L; ++l) { CHECK(moe_layer_destroy(lay[l]) == MOE_OK); delete arenas[l]; }
    CHECK(moe_ctx_destroy(ctx) == MOE_OK);
}

void error_paths()
{
    moe_ctx_t *ctx = nullptr;
    moe_ctx_config_t bad{4, 0, 64, 64, 2, MOE_CTX_HOST_ONLY, 1 << 16};
    CHECK(moe_ctx_create(&bad, nullptr, 0, nullptr, nullptr, &ctx) == MOE_EINVAL && !ctx);
    CHECK(moe_ctx_create(nullptr, nullptr, 0, nullptr, nullptr, &ctx) == MOE_EINVAL);
    CHECK(moe_ctx_create(&bad, nullptr, 0, nullptr, nullptr, nullptr) == MOE_EINVAL);
    CHECK(moe_ctx_destroy(nullptr) == MOE_OK && moe_layer_destroy(nullptr) == MOE_OK);
    CHECK(moe_layer_stats(nullptr, nullptr) == MOE_EINVAL && moe_layer_reset(nullptr) == MOE_EINVAL);
    CHECK(moe_layer_step(nullptr, nullptr, nullptr, 1, nullptr, nullptr, nullptr) == MOE_EINVAL);
    CHECK(moe_layer_step_noalloc(nullptr, nullptr, nullptr, 1, nullptr, nullptr, nullptr) == MOE_EINVAL);
    CHECK(moe_stack_step(nullptr, 0, nullptr, 1, nullptr, nullptr) == MOE_EINVAL);
    CHECK(moe_expert_blob_bytes(100, 64, 4, 64) == 0 && moe_expert_blob_bytes(64, 64, 5, 64) == 0);
    CHECK(moe_ctx_set_option(nullptr, "x", 1) == MOE_EINVAL);
    ctx = host_ctx(2, 4, 64, 64, 2, moe_expert_blob_bytes(64, 64, 4, 64));
    CHECK(moe_ctx_set_option(ctx, "no_such_option", 1) == MOE_EINVAL && moe_ctx_set_option(ctx, nullptr, 1) == MOE_EINVAL);
    CHECK(moe_ctx_profile_enable(ctx, 1) == MOE_ESTATE);
    moe_profile_t prof;
    CHECK(moe_ctx_profile_read(ctx, &prof) == MOE_ESTATE);
    float y[64];
    CHECK(moe_ctx_read_y(ctx, 1, 64, y) == MOE_ESTATE);
    moe_layer_config_t lc{64, 64, 4, 2, 4, 64, 2, 1, 0.f, 0, 0, 0};
    Arena host(moe_layer_host_bytes(&lc));
    std::vector<float> gate(4 * 64, 0.f);
    moe_layer_t *lay = nullptr;
    CHECK(moe_layer_create(ctx, &lc, gate.data(), nullptr, nullptr, host.p, &lay) == MOE_OK);
    int32_t idx[2] = {0, 4};
    CHECK(moe_layer_resolve(lay, nullptr, idx, 1, nullptr, nullptr) == MOE_EINVAL);     // expert 4 of 4
    idx[1] = 1;
    CHECK(moe_layer_resolve(lay, nullptr, idx, 5, nullptr, nullptr) == MOE_EINVAL);     // batch above the context's
    CHECK(moe_layer_resolve(lay, nullptr, nullptr, 1, nullptr, nullptr) == MOE_EINVAL);
    CHECK(moe_layer_step(lay, nullptr, (const uint16_t *)y, 1, (uint16_t *)y, nullptr, nullptr) == MOE_ESTATE);
    CHECK(moe_layer_step_noalloc(lay, nullptr, (const uint16_t *)y, 1, (uint16_t *)y, nullptr, nullptr) == MOE_ESTATE);
    CHECK(moe_layer_prefetch(lay, (const uint16_t *)y, 1, nullptr) == MOE_ESTATE);
    CHECK(moe_layer_set_prefetch(lay, 5) == MOE_EINVAL && moe_layer_set_flags(lay, 64) == MOE_EINVAL);
    uint8_t code; uint16_t a, b;
    CHECK(moe_layer_peek_weight(lay, 0, 0, 0, 0, &code, &a, &b) == MOE_ESTATE);           // not loaded yet
    CHECK(moe_layer_peek_weight(lay, 0, 3, 0, 0, &code, &a, &b) == MOE_EINVAL);
    CHECK(moe_layer_destroy(lay) == MOE_OK && moe_ctx_destroy(ctx) == MOE_OK);
}

}  // namespace

int main()
{
    std::mt19937 rng(20231217);
    const int fmts[5][2] = {{4, 32}, {4, 64}, {4, 128}, {3, 64}, {2, 16}};
    const int shapes[4][2] = {{64, 64}, {192, 320}, {256, 448}, {128, 1024}};
    int blobs = 0;
    for (auto &f : fmts)
        for (auto &sh : shapes)
            for (int R : {0, 2, 4, 8, 256}) {
                if (sh[0] % f[1] || sh[1] % f[1]) continue;
                pack_and_peek(sh[0], sh[1], f[0], f[1], R, rng);
                ++blobs;
            }
    for (unsigned seed = 0; seed < 60; ++seed) bookkeeping(1000 + seed);
    error_paths();
    std::printf("ok: %d blob layouts, 60 bookkeeping runs, error paths\n", blobs);
    return 0;
}
