// Decoding loops over an abstract per-model step interface: Algorithm 1
// (asynchronous draft and verify processes), synchronous speculative decoding
// and plain autoregressive decoding.  Host-only C++ with no GPU dependency, so
// the coordination logic can be exercised on the CPU (including under a thread
// sanitizer) with a stand-in backend.
#pragma once
#include <stdint.h>

#include <atomic>
#include <chrono>
#include <thread>
#include <vector>

namespace amusd {

struct StepBackend {
    virtual ~StepBackend() {}
    virtual int prefill(const int32_t* tokens, int n, int32_t* next) = 0;
    virtual int verify(int ctx_len, const int32_t* draft, int k, int32_t* accept_len, int32_t* next) = 0;
    virtual int draft_step(int32_t* token_out) = 0;
    virtual int rollback(int new_len) = 0;
    virtual int set_next(int32_t token) = 0;
    virtual int kv_len() const = 0;
    virtual int max_ctx() const = 0;
    virtual int vocab() const = 0;
};

struct LoopStats {
    int rounds = 0, rollbacks = 0, draft_steps = 0, accepted_total = 0;
    int accept_hist[17] = {0};
    double wall_ms = 0.0;
};

using Clock = std::chrono::steady_clock;
inline double ms_since(Clock::time_point t0) {
    return std::chrono::duration<double, std::milli>(Clock::now() - t0).count();
}

// Optional hook called around every shared-state access of run_async; tests
// use it to perturb the interleaving.  Must be set before the loop starts.
using JitterFn = void (*)(void* ctx, int site);

struct AsyncOptions {
    JitterFn jitter = nullptr;
    void* jitter_ctx = nullptr;
    double timeout_ms = 600000.0;
};

// Algorithm 1.  D[i] / V[i]: the draft's / the committed token at absolute
// position i.  p_d = number of valid entries of D (written by the draft thread
// only); p_v = verify cache length, tokens V[0..p_v] are committed (written by
// the verify thread only); R = rollback flag, raised by verify, cleared by
// draft.  A token buffer entry is published by the release-store of its
// counter (or of R) and read after the matching acquire-load.
inline int run_async(StepBackend& draft, StepBackend& verify, const int32_t* prompt, int P, int n_new, int k_max,
                     int32_t* out, LoopStats* stats, const AsyncOptions& opt = AsyncOptions()) {
    const int cap = verify.max_ctx() < draft.max_ctx() ? verify.max_ctx() : draft.max_ctx();
    if (P + 1 > cap) return -3;
    int rc;
    if (verify.kv_len() > 0 && (rc = verify.rollback(0))) return rc;
    if (draft.kv_len() > 0 && (rc = draft.rollback(0))) return rc;
    std::vector<int32_t> D((size_t)cap + 1, -1), V((size_t)cap + 1, -1);
    for (int i = 0; i < P; ++i) D[i] = V[i] = prompt[i];
    int32_t t = -1;
    if ((rc = verify.prefill(prompt, P, &t))) return rc;
    V[P] = t;
    if ((rc = draft.prefill(prompt, P, &t))) return rc;
    D[P] = t;
    std::atomic<int> p_d(P + 1), p_v(P), err(0);
    std::atomic<bool> R(false), done(false);
    int corr_pos = 0;
    int32_t corr_tok = -1;
    LoopStats st;
    const auto t0 = Clock::now();
    auto jit = [&](int site) {
        if (opt.jitter) opt.jitter(opt.jitter_ctx, site);
    };
    auto expired = [&] { return ms_since(t0) > opt.timeout_ms; };

    std::thread draft_thread([&] {
        int steps = 0;
        while (!done.load(std::memory_order_acquire) && !expired()) {
            jit(0);
            const int pd = p_d.load(std::memory_order_relaxed);
            if (pd < cap && draft.kv_len() < cap - 1 && draft.kv_len() == pd - 1) {
                int32_t tok = -1;
                const int e = draft.draft_step(&tok);      // one draft-model step: feeds D[pd-1], yields D[pd]
                if (e) { err.store(e); done.store(true, std::memory_order_release); break; }
                ++steps;
                D[pd] = tok;
                jit(1);
                p_d.store(pd + 1, std::memory_order_release);
            } else {
                std::this_thread::yield();
            }
            jit(2);
            if (R.load(std::memory_order_acquire)) {       // the verifier disagreed: truncate the draft cache to the corrected position
                const int c = corr_pos;
                int e = draft.rollback(c);
                if (!e) e = draft.set_next(corr_tok);
                if (e) { err.store(e); done.store(true, std::memory_order_release); break; }
                D[c] = corr_tok;
                p_d.store(c + 1, std::memory_order_release);
                jit(3);
                R.store(false, std::memory_order_release);
            }
        }
        st.draft_steps = steps;
    });

    // the verify side runs on the calling thread
    while (!done.load(std::memory_order_acquire) && !expired()) {
        jit(4);
        const int L = p_v.load(std::memory_order_relaxed);
        const int pd = p_d.load(std::memory_order_acquire);
        if (pd > L) {
            int k = pd - L;
            if (k > k_max) k = k_max;
            if (k > cap - L) k = cap - L;
            int32_t n = 0, nxt = -1;
            const int e = verify.verify(L, &D[L], k, &n, &nxt);   // one pass over the drafts published so far (at most k_max of them)
            if (e) { err.store(e); break; }
            for (int i = 0; i < n; ++i) V[L + i] = D[L + i];
            V[L + n] = nxt;
            ++st.rounds;
            st.accepted_total += n;
            ++st.accept_hist[n];
            jit(5);
            p_v.store(L + n, std::memory_order_release);
            if (n < k) {                                          // a draft was wrong: publish the correction, then the flag
                corr_pos = L + n;
                corr_tok = nxt;
                ++st.rollbacks;
                R.store(true, std::memory_order_release);
            }
        } else {
            std::this_thread::yield();
        }
        const int pv = p_v.load(std::memory_order_relaxed);
        if (pv + 1 - P >= n_new || pv + 1 >= cap) break;          // token budget reached
        while (R.load(std::memory_order_acquire) && !done.load(std::memory_order_acquire) && !expired()) {
            jit(6);
            std::this_thread::yield();                            // until the draft side has truncated its cache
        }
    }
    done.store(true, std::memory_order_release);
    draft_thread.join();
    st.wall_ms = ms_since(t0);
    if (stats) *stats = st;
    if (err.load()) return err.load();
    const int have = p_v.load() + 1 - P;
    if (have < n_new) return expired() ? -5 : -3;
    for (int i = 0; i < n_new; ++i) out[i] = V[P + i];
    return 0;
}

// Synchronous speculative decoding: a draft phase of k_max-1 steps, then one
// verify pass whose first row is the last committed token.
inline int run_sync(StepBackend& draft, StepBackend& verify, const int32_t* prompt, int P, int n_new, int k_max,
                    int32_t* out, LoopStats* stats) {
    const int cap = verify.max_ctx() < draft.max_ctx() ? verify.max_ctx() : draft.max_ctx();
    if (P + 1 > cap) return -3;
    int rc;
    if (verify.kv_len() > 0 && (rc = verify.rollback(0))) return rc;
    if (draft.kv_len() > 0 && (rc = draft.rollback(0))) return rc;
    std::vector<int32_t> V((size_t)cap + 1, -1), win(k_max);
    for (int i = 0; i < P; ++i) V[i] = prompt[i];
    int32_t t = -1;
    if ((rc = verify.prefill(prompt, P, &t))) return rc;
    V[P] = t;
    if ((rc = draft.prefill(prompt, P, &t))) return rc;
    LoopStats st;
    const auto t0 = Clock::now();
    int L = P;                                   // verify cache length; V[0..L] committed
    while (L + 1 - P < n_new && L + 1 < cap) {
        int k = k_max < cap - L ? k_max : cap - L;
        // draft cache holds V[0..L); feed V[L], then its own guesses
        if ((rc = draft.set_next(V[L]))) return rc;
        win[0] = V[L];
        for (int j = 1; j < k; ++j) {
            if ((rc = draft.draft_step(&win[j]))) return rc;
            ++st.draft_steps;
        }
        int32_t n = 0, nxt = -1;
        if ((rc = verify.verify(L, win.data(), k, &n, &nxt))) return rc;
        for (int i = 0; i < n; ++i) V[L + i] = win[i];
        V[L + n] = nxt;
        ++st.rounds;
        st.accepted_total += n;
        ++st.accept_hist[n];
        if (n < k) ++st.rollbacks;
        L += n;
        // the draft fed win[0..k-2]; keep the rows that were accepted
        const int keep = L < draft.kv_len() ? L : draft.kv_len();
        if ((rc = draft.rollback(keep))) return rc;
        if (draft.kv_len() < L) {                // all k accepted: the draft never fed win[k-1]
            if ((rc = draft.set_next(V[draft.kv_len()]))) return rc;
            int32_t dummy;
            if ((rc = draft.draft_step(&dummy))) return rc;
            ++st.draft_steps;
        }
    }
    st.wall_ms = ms_since(t0);
    if (stats) *stats = st;
    if (L + 1 - P < n_new) return -3;
    for (int i = 0; i < n_new; ++i) out[i] = V[P + i];
    return 0;
}

// Autoregressive decoding: prefill, then one single-row pass per token.
inline int run_greedy(StepBackend& m, const int32_t* prompt, int P, int n_new, int32_t* out, LoopStats* stats) {
    if (P + n_new > m.max_ctx() + 1) return -3;
    int rc;
    if (m.kv_len() > 0 && (rc = m.rollback(0))) return rc;
    int32_t t = -1;
    if ((rc = m.prefill(prompt, P, &t))) return rc;
    LoopStats st;
    const auto t0 = Clock::now();
    out[0] = t;
    for (int i = 1; i < n_new; ++i) {
        if ((rc = m.draft_step(&t))) return rc;
        ++st.draft_steps;
        out[i] = t;
    }
    st.wall_ms = ms_since(t0);
    if (stats) *stats = st;
    return 0;
}

}  // namespace amusd
