// CPU test of the decoding loops (Algorithm 1 and the two baselines) against a
// stand-in backend with a known answer.  No GPU, no HIP: built with g++ and run
// under ThreadSanitizer by tests/test_loops_cpu.py.
//
// Stand-in model: the greedy token after a prefix is a hash of the whole prefix,
// so any wrong token in the cache changes everything after it.  The draft model
// agrees with the verify model except where hash % 3 == 0.
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <random>
#include <vector>

#include "../../paper_2410_17375_amd/csrc/amusd_loops.h"

using namespace amusd;

struct FakeModel final : StepBackend {
    int V, cap, flavour;
    std::vector<int32_t> cache;        // tokens whose keys/values are "cached"
    std::vector<int32_t> greedy_at;    // greedy_at[p]: model's token for position p, -1 unknown
    int32_t p_next = -1;
    long passes = 0;
    FakeModel(int vocab, int max_ctx, int flav) : V(vocab), cap(max_ctx), flavour(flav), greedy_at(max_ctx + 2, -1) {}
    int32_t next_of(const std::vector<int32_t>& pre, size_t n) const {
        uint64_t h = 1469598103934665603ull;
        for (size_t i = 0; i < n; ++i) { h ^= (uint64_t)(pre[i] + 1); h *= 1099511628211ull; }
        int32_t t = (int32_t)(h % (uint64_t)V);
        if (flavour && (h >> 20) % 3 == 0) t = (t + 1) % V;     // the draft model disagrees here
        return t;
    }
    int prefill(const int32_t* t, int n, int32_t* next) override {
        if ((int)cache.size() + n > cap) return -3;
        for (int i = 0; i < n; ++i) { cache.push_back(t[i]); greedy_at[cache.size()] = next_of(cache, cache.size()); }
        p_next = greedy_at[cache.size()];
        if (next) *next = p_next;
        return 0;
    }
    int verify(int L, const int32_t* d, int k, int32_t* acc, int32_t* next) override {
        if (L < 0 || L > (int)cache.size()) return -2;
        if (L + k > cap) return -3;
        if (greedy_at[L] < 0) return -5;
        ++passes;
        cache.resize(L);
        std::vector<int32_t> g(k);
        for (int j = 0; j < k; ++j) { cache.push_back(d[j]); g[j] = next_of(cache, cache.size()); greedy_at[L + j + 1] = g[j]; }
        int n = 0;
        while (n < k && d[n] == (n ? g[n - 1] : greedy_at[L])) ++n;
        *acc = n;
        *next = n < k ? (n ? g[n - 1] : greedy_at[L]) : g[k - 1];
        cache.resize(L + n);
        p_next = *next;
        return 0;
    }
    int draft_step(int32_t* out) override {
        if (p_next < 0) return -5;
        if ((int)cache.size() + 1 > cap) return -3;
        cache.push_back(p_next);
        p_next = next_of(cache, cache.size());
        greedy_at[cache.size()] = p_next;
        *out = p_next;
        return 0;
    }
    int rollback(int n) override {
        if (n < 0 || n > (int)cache.size()) return -2;
        cache.resize(n);
        p_next = greedy_at[n];
        return 0;
    }
    int set_next(int32_t t) override { p_next = t; greedy_at[cache.size()] = t; return 0; }
    int kv_len() const override { return (int)cache.size(); }
    int max_ctx() const override { return cap; }
    int vocab() const override { return V; }
};

struct Jit { std::mt19937 rng; };
static void jitter(void* ctx, int) {
    // called from both threads: keep per-thread generators
    thread_local std::mt19937 r(std::random_device{}());
    (void)ctx;
    const unsigned x = r() % 64;
    if (x == 0) std::this_thread::sleep_for(std::chrono::microseconds(r() % 200));
    else if (x < 8) std::this_thread::yield();
}

int main(int argc, char** argv) {
    const int trials = argc > 1 ? atoi(argv[1]) : 20;
    const int V = 97, cap = 400, P = 23, N = 120;
    std::vector<int32_t> prompt(P);
    for (int i = 0; i < P; ++i) prompt[i] = (i * 31 + 7) % V;
    FakeModel ref(V, cap, 0);
    std::vector<int32_t> want(N), got(N);
    LoopStats st;
    if (run_greedy(ref, prompt.data(), P, N, want.data(), &st)) { printf("greedy failed\n"); return 1; }
    int bad = 0;
    for (int k = 1; k <= 16; k += 3) {
        FakeModel d(V, cap, 1), v(V, cap, 0);
        if (run_sync(d, v, prompt.data(), P, N, k, got.data(), &st) || got != want) { printf("sync k=%d mismatch\n", k); ++bad; }
        if (st.accepted_total < st.rounds && k > 1) { printf("sync k=%d: every window's first row must match\n", k); ++bad; }
    }
    for (int t = 0; t < trials; ++t) {
        const int k = 1 + t % 16;
        FakeModel d(V, cap, t % 4 == 3 ? 0 : 1), v(V, cap, 0);   // every 4th trial: draft == verify (no rollbacks needed)
        AsyncOptions opt;
        opt.jitter = jitter;
        opt.timeout_ms = 60000.0;
        const int rc = run_async(d, v, prompt.data(), P, N, k, got.data(), &st, opt);
        if (rc || got != want) { printf("async trial %d (k=%d) rc=%d mismatch\n", t, k, rc); ++bad; }
        int hist = 0;
        for (int i = 0; i <= 16; ++i) hist += st.accept_hist[i];
        if (hist != st.rounds) { printf("async trial %d: histogram does not add up\n", t); ++bad; }
        if (t % 4 == 3 && st.rollbacks != 0) { printf("async trial %d: twin draft must never be rolled back\n", t); ++bad; }
    }
    // capacity: the loop stops with an error instead of overrunning the caches
    {
        FakeModel d(V, 40, 1), v(V, 40, 0);
        const int rc = run_async(d, v, prompt.data(), P, N, 4, got.data(), &st);
        if (rc == 0) { printf("capacity overrun not reported\n"); ++bad; }
    }
    printf(bad ? "FAILED %d\n" : "OK %d\n", bad);
    return bad ? 1 : 0;
}
