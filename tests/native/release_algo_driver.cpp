// CPU exercise of the protocol by which work-groups share an agent-scope release
// (csrc/shm_release_algo.hpp): threads play the groups' leaders, std::atomic plays the word, and a
// logical clock orders arrivals, write-backs and returns.  The property that makes the protocol a
// quiet: every call returns only after a write-back that BEGAN after the call's arrival has FINISHED.
// It is checked for every call under heavy contention; the same harness run on a protocol with a
// planted mistake (waiting for the write-back already under way instead of the next one) must report
// violations, which shows that the check can fail.  Prints "ok" and exits 0 if every check holds.
#include <algorithm>
#include <atomic>
#include <cstdint>
#include <cstdio>
#include <random>
#include <thread>
#include <vector>

#include "shm_release_algo.hpp"

namespace {

std::atomic<uint64_t> g_clock{1};
uint64_t tick() { return g_clock.fetch_add(1, std::memory_order_seq_cst); }

struct flush_record {
    uint64_t begin, end;
};

struct host_ops {
    std::atomic<unsigned long long> *word;
    std::vector<flush_record> *flushes;      // this thread's write-backs
    int work;                                // length of a write-back, in spins
    unsigned long long fetch_or_lock() { return word->fetch_or(1ull, std::memory_order_relaxed); }
    unsigned long long load() { return word->load(std::memory_order_relaxed); }
    void store(unsigned long long v) { word->store(v, std::memory_order_relaxed); }
    void write_back()
    {
        flush_record r;
        r.begin = tick();
        for (volatile int i = 0; i < work; ++i) {
        }
        r.end = tick();
        flushes->push_back(r);
    }
    void pause() { std::this_thread::yield(); }
};

// The planted mistake: a caller that finds the lock held is content with the write-back under way.
template <typename Ops>
void broken_algo(Ops &ops, int spin_limit)
{
    unsigned long long v = ops.fetch_or_lock();
    if (!(v & 1ull)) {
        ops.write_back();
        ops.store(v + 2ull);
        return;
    }
    const unsigned long long need = (v >> 1) + 1ull;       // should be + 2
    for (int spin = 0; spin < spin_limit; ++spin) {
        ops.pause();
        if ((ops.load() >> 1) >= need) return;
    }
    ops.write_back();
}

struct call_record {
    uint64_t arrive, ret;
};

struct result {
    uint64_t calls = 0, violations = 0, flushes = 0, stuck_lock = 0;
};

template <typename Algo>
result run(Algo algo, int n_threads, int calls_per_thread, int work)
{
    std::atomic<unsigned long long> word{0};
    std::vector<std::vector<flush_record>> flushes(n_threads);
    std::vector<std::vector<call_record>> calls(n_threads);
    std::vector<std::thread> threads;
    for (int t = 0; t < n_threads; ++t)
        threads.emplace_back([&, t] {
            std::mt19937 rng(1234u + t);
            host_ops ops{&word, &flushes[t], work};
            calls[t].reserve(calls_per_thread);
            for (int i = 0; i < calls_per_thread; ++i) {
                const int idle = static_cast<int>(rng() % 64u) * (rng() % 8u == 0 ? 40 : 1);      // bursts and gaps
                for (volatile int k = 0; k < idle; ++k) {
                }
                call_record c;
                c.arrive = tick();                 // "my stores are acknowledged"
                algo(ops, 1 << 22);
                c.ret = tick();
                calls[t].push_back(c);
            }
        });
    for (auto &th : threads) th.join();
    std::vector<flush_record> all;
    for (auto &f : flushes) all.insert(all.end(), f.begin(), f.end());
    std::sort(all.begin(), all.end(), [](const flush_record &a, const flush_record &b) { return a.begin < b.begin; });
    // suffix minimum of end over flushes sorted by begin: the earliest finish among those begun after x
    std::vector<uint64_t> best_end(all.size() + 1, UINT64_MAX);
    for (size_t i = all.size(); i-- > 0;) best_end[i] = std::min(best_end[i + 1], all[i].end);
    result r;
    r.flushes = all.size();
    for (auto &per_thread : calls)
        for (const call_record &c : per_thread) {
            ++r.calls;
            const size_t i = std::upper_bound(all.begin(), all.end(), c.arrive,
                                              [](uint64_t x, const flush_record &f) { return x < f.begin; }) - all.begin();
            if (best_end[i] >= c.ret) ++r.violations;
        }
    r.stuck_lock = word.load() & 1ull;
    // the count in the word is the number of write-backs published by lock holders
    return r;
}

}  // namespace

int main()
{
    int failures = 0;
    auto good = [](host_ops &ops, int limit) { shm_release_shared_algo(ops, limit); };
    auto bad = [](host_ops &ops, int limit) { broken_algo(ops, limit); };
    for (int n_threads : {2, 4, 16}) {
        for (int work : {0, 200, 5000}) {
            const result r = run(good, n_threads, 20000, work);
            std::printf("protocol: %2d threads, write-back %4d spins: %llu calls, %llu write-backs, %llu violations, lock %s\n", n_threads,
                        work, (unsigned long long)r.calls, (unsigned long long)r.flushes, (unsigned long long)r.violations,
                        r.stuck_lock ? "STUCK" : "clear");
            if (r.violations != 0 || r.stuck_lock != 0 || r.flushes == 0 || r.flushes > r.calls) ++failures;
        }
    }
    // sharing must actually happen under contention: far fewer write-backs than calls
    {
        const result r = run(good, 16, 20000, 5000);
        if (r.flushes * 2 > r.calls) {
            std::printf("no sharing: %llu write-backs for %llu calls\n", (unsigned long long)r.flushes, (unsigned long long)r.calls);
            ++failures;
        }
    }
    // the check itself: the planted mistake must be noticed
    {
        uint64_t seen = 0;
        for (int rep = 0; rep < 5 && seen == 0; ++rep) seen += run(bad, 16, 20000, 5000).violations;
        std::printf("planted mistake: %llu violations noticed\n", (unsigned long long)seen);
        if (seen == 0) ++failures;
    }
    if (failures) {
        std::printf("%d failures\n", failures);
        return 1;
    }
    std::printf("ok\n");
    return 0;
}
