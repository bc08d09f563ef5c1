// Minimal host-side parallel loop (std::thread); used by the offline paths only.
#pragma once
#include <algorithm>
#include <atomic>
#include <cstdint>
#include <cstdlib>
#include <thread>
#include <vector>

namespace lqer {

inline int host_threads() {
    static int n = [] {
        int v = 0;
        if (const char* e = std::getenv("LQER_HOST_THREADS")) v = std::atoi(e);
        if (v <= 0) v = (int)std::thread::hardware_concurrency();
        if (v <= 0) v = 1;
        return std::min(v, 64);
    }();
    return n;
}

// Calls fn(i) for every i in [0, n), dynamically scheduled in chunks over the host threads.
template <class F>
void parallel_for(int64_t n, F&& fn, int64_t chunk = 1) {
    const int nt = (int)std::min<int64_t>(host_threads(), (n + chunk - 1) / chunk);
    if (nt <= 1) {
        for (int64_t i = 0; i < n; ++i) fn(i);
        return;
    }
    std::atomic<int64_t> next{0};
    auto work = [&] {
        for (;;) {
            const int64_t b = next.fetch_add(chunk);
            if (b >= n) break;
            const int64_t e = std::min(n, b + chunk);
            for (int64_t i = b; i < e; ++i) fn(i);
        }
    };
    std::vector<std::thread> th;
    th.reserve(nt - 1);
    for (int t = 1; t < nt; ++t) th.emplace_back(work);
    work();
    for (auto& t : th) t.join();
}

}  // namespace lqer
