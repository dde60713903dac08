// Page bookkeeping of one model's paged KV cache: which physical pages every row (sequence, or candidate
// lane) names, the free list, and how many names each page has.  Host-only and free of HIP calls, so that
// a CPU build with sanitizers can drive it through reserve / roll back / share / exhaust sequences
// (tests/host/pages_driver.cpp).  The table's storage belongs to the caller (the library keeps it in
// pinned memory, from where it is copied to the device whenever `bt_dirty` is set).
//
// Contract: row b names n_pages[b] pages, logical page i at bt_host[b * max_pages + i], -1 beyond; a page
// is in the free list iff no row names it; ref[p] is the number of names of p (above 1 only while the
// candidates of a Best-of-N step share a committed context).  Pages are handed out in LIFO order.
#pragma once
#include <string>
#include <vector>

struct PageTable {
    int pool_pages = 0, max_pages = 0, n_rows = 0;
    std::vector<int> free_list;
    std::vector<int> ref;
    int* bt_host = nullptr;      // [n_rows][max_pages], caller-owned
    std::vector<int> n_pages;
    bool bt_dirty = false;

    void init_pages(int rows, int max_pages_, int pool_pages_, int* storage) {
        n_rows = rows; max_pages = max_pages_; pool_pages = pool_pages_; bt_host = storage;
        free_list.resize(pool_pages);
        for (int i = 0; i < pool_pages; ++i) free_list[i] = pool_pages - 1 - i;   // pop_back hands out 0,1,2,...
        ref.assign(pool_pages, 0);
        for (size_t i = 0; i < (size_t)rows * max_pages; ++i) bt_host[i] = -1;
        n_pages.assign(rows, 0);
        bt_dirty = true;
    }
    // row b grows to `need` pages; false (row unchanged beyond what it got) when the pool runs out
    bool ensure(int b, int need) {
        if (need > max_pages) return false;
        while (n_pages[b] < need) {
            if (free_list.empty()) return false;
            const int pg = free_list.back();
            free_list.pop_back();
            ref[pg] = 1;
            bt_host[(size_t)b * max_pages + n_pages[b]++] = pg;
            bt_dirty = true;
        }
        return true;
    }
    // row b keeps its first `keep` pages; a page returns to the pool when its last name goes
    void trim(int b, int keep) {
        while (n_pages[b] > keep) {
            int& e = bt_host[(size_t)b * max_pages + --n_pages[b]];
            if (--ref[e] == 0) free_list.push_back(e);
            e = -1;
            bt_dirty = true;
        }
    }
    // the next logical page of row b becomes another name of physical page pg
    void share(int b, int pg) {
        ++ref[pg];
        bt_host[(size_t)b * max_pages + n_pages[b]++] = pg;
        bt_dirty = true;
    }
    // the invariants above; on failure `why` says which one broke
    bool consistent(std::string* why = nullptr) const {
        std::vector<int> names(pool_pages, 0);
        auto bad = [&](const char* t) { if (why) *why = t; return false; };
        for (int b = 0; b < n_rows; ++b) {
            if (n_pages[b] < 0 || n_pages[b] > max_pages) return bad("n_pages out of range");
            for (int i = 0; i < max_pages; ++i) {
                const int e = bt_host[(size_t)b * max_pages + i];
                if (i < n_pages[b]) {
                    if (e < 0 || e >= pool_pages) return bad("table entry outside the pool");
                    ++names[e];
                } else if (e != -1) return bad("entry beyond n_pages is not -1");
            }
        }
        std::vector<char> is_free(pool_pages, 0);
        for (int p : free_list) {
            if (p < 0 || p >= pool_pages) return bad("free-list entry outside the pool");
            if (is_free[p]) return bad("page twice in the free list");
            is_free[p] = 1;
        }
        for (int p = 0; p < pool_pages; ++p) {
            if (names[p] != ref[p] && !(is_free[p] && names[p] == 0)) return bad("reference count differs from the number of names");
            if ((names[p] == 0) != (is_free[p] != 0)) return bad("a page is neither named nor free, or both");
        }
        return true;
    }
};

// Rows of a decode iteration that serves n_act of B sequences, or 0 when one row per sequence is as cheap.
// The sizes are those at which the matrix kernels change: up to 8 rows the exact count (single-row and
// few-row vector kernels), 32 and 64 (one or two MFMA row tiles of the weight-streaming kernels), then whole
// 128-row tiles.
inline int packed_rows(int n_act, int B) {
    const int r = n_act <= 8 ? n_act : n_act <= 32 ? 32 : n_act <= 64 ? 64 : (n_act + 127) / 128 * 128;
    return r < B ? r : 0;
}
// The row map of such an iteration: the taking-part sequences in ascending order, then -1 for the unused rows.
inline void fill_packed_rows(const std::vector<int>& seqs, int rows, int* row_seq) {
    int r = 0;
    for (int b : seqs) row_seq[r++] = b;
    for (; r < rows; ++r) row_seq[r] = -1;
}
