// Host-only exercise of the reverse-offload proxy thread (paper section "Synchronization with
// Host"): CPU threads play the GPU senders and speak the ring protocol -- slot by fetch-and-add,
// four tagged 16-byte quarters per 64-byte message (written in a scrambled order, as separate
// stores may land), completion words allocated independently of slots, flow control against the
// consumed count -- while the real proxy thread serves them.  No GPU and no HSA call is involved:
// with an empty engine list a copy request is answered at once.  Prints "ok" and exits 0 if every
// check holds.
#include <atomic>
#include <cstdio>
#include <cstdlib>
#include <thread>
#include <vector>

#include "shm_proxy.hpp"

namespace {

struct sender_side {
    shm_offload_shared *sh;
    std::atomic<uint64_t> head{0}, comp_head{0};
};

int failures = 0;
#define CHECK(cond)                                                         \
    do {                                                                    \
        if (!(cond)) {                                                      \
            std::printf("check failed, line %d: %s\n", __LINE__, #cond);    \
            ++failures;                                                     \
        }                                                                   \
    } while (0)

// Returns false if the ring stayed full or the answer did not come within ten seconds.
bool send(sender_side &s, uint32_t op, uint32_t pe, bool want_completion, unsigned scramble)
{
    const auto t0 = std::chrono::steady_clock::now();
    auto late = [&] { return std::chrono::duration<double>(std::chrono::steady_clock::now() - t0).count() > 10.0; };
    const uint64_t idx = s.head.fetch_add(1);
    uint32_t ticket = SHM_OFFLOAD_NO_COMPLETION;
    if (want_completion) {
        ticket = static_cast<uint32_t>(s.comp_head.fetch_add(1));
        if (ticket == SHM_OFFLOAD_NO_COMPLETION) ticket = static_cast<uint32_t>(s.comp_head.fetch_add(1));
    }
    while (idx - __atomic_load_n(&s.sh->consumed, __ATOMIC_ACQUIRE) >= SHM_OFFLOAD_SLOTS) {
        if (late()) return false;
        std::this_thread::yield();
    }
    const uint32_t tag = static_cast<uint32_t>(idx / SHM_OFFLOAD_SLOTS) + 1u;
    uint32_t m[16] = {op, pe, ticket, tag, 0x1000, 0, 0, tag, 0x2000, 0, 0, tag, 64, 0, 0, tag};
    uint32_t *slot = s.sh->ring[idx & (SHM_OFFLOAD_SLOTS - 1)];
    for (unsigned k = 0; k < 4; ++k) {
        const unsigned q = (k + scramble) & 3;
        for (unsigned w = 0; w < 3; ++w) slot[4 * q + w] = m[4 * q + w];
        __atomic_store_n(&slot[4 * q + 3], tag, __ATOMIC_RELEASE);      // the tag of a quarter lands after its payload
        if ((idx & 255) == 0) std::this_thread::yield();      // now and then leave a message half-written for a while
    }
    if (!want_completion) return true;
    const uint32_t *word = &s.sh->completion[ticket & (SHM_OFFLOAD_COMPLETIONS - 1)];
    const uint32_t want = ticket / SHM_OFFLOAD_COMPLETIONS + 1u;
    while (__atomic_load_n(word, __ATOMIC_ACQUIRE) != want) {
        if (late()) return false;
        std::this_thread::yield();
    }
    return true;
}

}  // namespace

int main()
{
    void *mem = nullptr;
    if (posix_memalign(&mem, 4096, sizeof(shm_offload_shared)) != 0) return 2;
    memset(mem, 0, sizeof(shm_offload_shared));
    sender_side s;
    s.sh = static_cast<shm_offload_shared *>(mem);

    shm_proxy proxy;
    CHECK(!proxy.running());
    proxy.start(s.sh, hsa_agent_t{}, std::vector<uint32_t>{}, 4);
    CHECK(proxy.running());

    // one round trip of every kind, including a PE the proxy does not know
    CHECK(send(s, SHM_OFFLOAD_NOP, 0, true, 0));
    CHECK(send(s, SHM_OFFLOAD_QUIET, 3, true, 1));
    CHECK(send(s, SHM_OFFLOAD_COPY, 1, true, 2));          // no engines: answered without a transfer
    CHECK(send(s, SHM_OFFLOAD_NOP, 77, true, 3));
    CHECK(send(s, 12345u, 2, true, 0));                    // unknown request kinds are answered too
    CHECK(proxy.requests() == 5);
    CHECK(proxy.copies() == 0);

    // four senders, blocking and fire-and-forget mixed: the 4096-slot ring wraps several times and
    // the completion words are reused (65536 of them, 4 x 20000 blocking requests)
    constexpr int kSenders = 4, kPerSender = 40000;
    std::atomic<int> bad{0};
    std::vector<std::thread> threads;
    for (int t = 0; t < kSenders; ++t)
        threads.emplace_back([&, t] {
            for (int i = 0; i < kPerSender; ++i)
                if (!send(s, (i % 3 == 0) ? SHM_OFFLOAD_QUIET : SHM_OFFLOAD_NOP, static_cast<uint32_t>(t), (i & 1) == 0, static_cast<unsigned>(i + t)))
                    bad.fetch_add(1);
        });
    for (auto &t : threads) t.join();
    CHECK(bad.load() == 0);
    const uint64_t total = 5 + static_cast<uint64_t>(kSenders) * kPerSender;
    CHECK(s.head.load() == total);

    // the host's quiet: everything sent so far is taken, nothing is in flight
    CHECK(proxy.wait_idle(total, -1, 10.0));
    CHECK(proxy.wait_idle(total, 2, 10.0));
    CHECK(proxy.requests() == total);
    CHECK(!proxy.wait_idle(total + 1, -1, 0.05));          // a message nobody has sent is never taken
    CHECK(proxy.take_failed() == 0);

    // stop takes what is still in the ring first
    for (int i = 0; i < 1000; ++i) CHECK(send(s, SHM_OFFLOAD_NOP, 1, false, static_cast<unsigned>(i)));
    proxy.stop(s.head.load());
    CHECK(!proxy.running());
    CHECK(proxy.requests() == total + 1000);

    // restart: ring and counters begin again
    memset(mem, 0, sizeof(shm_offload_shared));
    s.head = 0;
    s.comp_head = 0;
    proxy.start(s.sh, hsa_agent_t{}, std::vector<uint32_t>{}, 2);
    CHECK(send(s, SHM_OFFLOAD_NOP, 1, true, 2));
    CHECK(proxy.requests() == 1);
    proxy.stop(1);
    proxy.stop();                                          // a second stop is harmless

    free(mem);
    if (failures) return 1;
    std::printf("ok\n");
    return 0;
}
