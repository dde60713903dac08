// CPU driver for the page bookkeeping of the paged KV cache (csrc/pages.h), meant to be built with
// -fsanitize=address,undefined: random reserve / roll back / share / release sequences in the patterns
// the step loops use, with the table's invariants checked after every operation and the contents
// compared with a plain model (a set of names per page).  Exit status 0 = every check held.
#include <cstdio>
#include <cstdlib>
#include <map>
#include <random>
#include <set>
#include <vector>

#include "pages.h"

#define REQUIRE(cond)                                                              \
    do {                                                                           \
        if (!(cond)) { std::printf("FAILED %s (line %d)\n", #cond, __LINE__); std::exit(1); } \
    } while (0)

static void check(const PageTable& t) {
    std::string why;
    if (!t.consistent(&why)) { std::printf("inconsistent: %s\n", why.c_str()); std::exit(1); }
}
static int ceil_div(int a, int b) { return (a + b - 1) / b; }

// the reserve / roll back pattern of one reasoning step of the accept-or-regenerate loop
static void rsd_pattern(unsigned seed) {
    std::mt19937 rng(seed);
    const int B = 5, page = 16, max_ctx = 400, cap = 24;
    const int max_pages = ceil_div(max_ctx, page), pool = 3 + (int)(rng() % (B * max_pages));
    std::vector<int> storage((size_t)B * max_pages);
    PageTable t;
    t.init_pages(B, max_pages, pool, storage.data());
    check(t);
    std::vector<int> kv(B, 0), ctx(B);
    for (int b = 0; b < B; ++b) ctx[b] = 1 + (int)(rng() % 60);
    for (int step = 0; step < 40; ++step) {
        // reserve room for a whole step up front; on exhaustion every row goes back to what it holds tokens for
        bool ok = true;
        for (int b = 0; b < B && ok; ++b) ok = t.ensure(b, ceil_div(std::min(ctx[b] + cap, max_ctx), page));
        check(t);
        if (!ok) {
            for (int b = 0; b < B; ++b) t.trim(b, ceil_div(kv[b], page));
            check(t);
            for (int b = 0; b < B; ++b) REQUIRE(t.n_pages[b] == ceil_div(kv[b], page));
            // free some rows entirely (sequences that finished) and go on
            const int b = (int)(rng() % B);
            t.trim(b, 0); kv[b] = 0; ctx[b] = 1 + (int)(rng() % 30);
            check(t);
            continue;
        }
        for (int b = 0; b < B; ++b) {
            const int grown = std::min(max_ctx, ctx[b] + 1 + (int)(rng() % cap));
            const bool accept = rng() % 2;
            if (accept) { ctx[b] = grown; kv[b] = grown - 1; }      // the step stays: cache up to the newest token
            else kv[b] = std::min(kv[b], ctx[b]);                    // rolled back: nothing beyond the old context
            t.trim(b, ceil_div(kv[b], page));
            check(t);
            REQUIRE(t.n_pages[b] == ceil_div(kv[b], page));
        }
    }
    for (int b = 0; b < B; ++b) t.trim(b, 0);
    check(t);
    REQUIRE((int)t.free_list.size() == pool);
}

// the fork / choose / release pattern of a Best-of-N step: candidates name the committed full pages,
// own their step's pages, and all but the chosen one give everything back
static void bon_pattern(unsigned seed) {
    std::mt19937 rng(seed);
    const int S = 3, N = 4, B = S * N, page = 16, max_ctx = 300, cap = 20;
    const int max_pages = ceil_div(max_ctx, page), pool = 8 + (int)(rng() % (B * max_pages));
    std::vector<int> storage((size_t)B * max_pages);
    PageTable t;
    t.init_pages(B, max_pages, pool, storage.data());
    std::vector<int> canon(S), ctx(S);
    for (int s = 0; s < S; ++s) { canon[s] = s * N; ctx[s] = 2 + (int)(rng() % 50); }
    for (int step = 0; step < 30; ++step) {
        bool ok = true;
        for (int s = 0; s < S && ok; ++s) ok = t.ensure(canon[s], ceil_div(ctx[s], page));
        std::vector<int> held(B, 0);
        for (int s = 0; s < S && ok; ++s) {
            const int L0 = canon[s], full = ctx[s] / page, need = ceil_div(std::min(ctx[s] + cap, max_ctx), page);
            for (int n = 0; n < N && ok; ++n) {
                const int L = s * N + n;
                if (L != L0) {
                    t.trim(L, 0);
                    for (int i = 0; i < full; ++i) t.share(L, t.bt_host[(size_t)L0 * max_pages + i]);
                    if (ctx[s] % page) ok = t.ensure(L, full + 1);      // the page that gets copied
                    if (ok) {
                        for (int i = 0; i < full; ++i) REQUIRE(t.bt_host[(size_t)L * max_pages + i] == t.bt_host[(size_t)L0 * max_pages + i]);
                        if (ctx[s] % page) REQUIRE(t.bt_host[(size_t)L * max_pages + full] != t.bt_host[(size_t)L0 * max_pages + full]);
                    }
                }
                ok = ok && t.ensure(L, need);
                check(t);
            }
        }
        if (!ok) {       // exhausted: candidates release everything, committed rows keep their context
            for (int s = 0; s < S; ++s)
                for (int n = 0; n < N; ++n) t.trim(s * N + n, s * N + n == canon[s] ? ceil_div(ctx[s], page) : 0);
            check(t);
            int used = 0;
            for (int s = 0; s < S; ++s) used += t.n_pages[canon[s]];
            REQUIRE(used + (int)t.free_list.size() == pool);
            const int s = (int)(rng() % S);      // a sequence ends and frees its pages
            t.trim(canon[s], 0); ctx[s] = 2 + (int)(rng() % 30);
            check(t);
            continue;
        }
        for (int s = 0; s < S; ++s) {
            const int w = (int)(rng() % N), Lw = s * N + w;
            const int grown = std::min(max_ctx, ctx[s] + 1 + (int)(rng() % cap));
            canon[s] = Lw;
            for (int n = 0; n < N; ++n) if (s * N + n != Lw) t.trim(s * N + n, 0);
            t.trim(Lw, ceil_div(grown, page));
            ctx[s] = grown;
            check(t);
            for (int i = 0; i < t.n_pages[Lw]; ++i) REQUIRE(t.ref[t.bt_host[(size_t)Lw * max_pages + i]] == 1);
            if (ctx[s] >= max_ctx) { t.trim(Lw, 0); ctx[s] = 2 + (int)(rng() % 30); }
        }
    }
    for (int b = 0; b < B; ++b) t.trim(b, 0);
    check(t);
    REQUIRE((int)t.free_list.size() == pool);
}

int main() {
    // edge cases: zero-page requests, a request beyond a row's table, an exhausted pool, LIFO order
    {
        std::vector<int> storage(2 * 4);
        PageTable t;
        t.init_pages(2, 4, 5, storage.data());
        REQUIRE(t.ensure(0, 0) && t.n_pages[0] == 0);
        REQUIRE(!t.ensure(0, 5));                        // more than the row's table holds
        REQUIRE(t.ensure(0, 3) && t.bt_host[0] == 0 && t.bt_host[1] == 1 && t.bt_host[2] == 2);
        REQUIRE(!t.ensure(1, 3) && t.n_pages[1] == 2);   // the pool had two pages left
        check(t);
        t.trim(1, 0);
        REQUIRE(t.ensure(1, 1) && t.bt_host[4] == 3);    // the page returned last is handed out first
        t.trim(0, 1); t.trim(0, 1);                      // trimming to the current size does nothing
        check(t);
        REQUIRE((int)t.free_list.size() == 3);
    }
    // packed rows of a partial stage: never fewer rows than sequences, never as many as the batch, one of the
    // sizes the matrix kernels distinguish, monotone in the number of sequences; the map lists the sequences
    // in order and marks the rest unused
    for (int B : {1, 2, 4, 8, 9, 16, 33, 64, 65, 192, 256, 300}) {
        int last = 0;
        for (int n = 1; n <= B; ++n) {
            const int r = packed_rows(n, B);
            REQUIRE(r == 0 || (r >= n && r < B));
            REQUIRE(r == 0 || r <= 8 || r == 32 || r == 64 || r % 128 == 0);
            if (r && last) REQUIRE(r >= last);
            if (n <= 8 && n < B) REQUIRE(r == n);
            if (n == B) REQUIRE(r == 0);
            if (r) last = r;
            if (r) {
                std::vector<int> seqs, map(r, 12345);
                for (int b = 0; b < B && (int)seqs.size() < n; ++b) if ((b * 7 + n) % 3 != 0 || B - b <= n - (int)seqs.size()) seqs.push_back(b);
                REQUIRE((int)seqs.size() == n);
                fill_packed_rows(seqs, r, map.data());
                for (int i = 0; i < r; ++i) REQUIRE(map[i] == (i < n ? seqs[i] : -1));
            }
        }
    }
    for (unsigned seed = 1; seed <= 300; ++seed) { rsd_pattern(seed); bon_pattern(seed); }
    std::printf("pages ok\n");
    return 0;
}
