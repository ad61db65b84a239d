// Reverse offload: a GPU thread asks the host to do something it cannot do itself -- here, start a
// copy engine -- through a lock-free ring in pinned host memory (paper section "Synchronization
// with Host").  The properties the paper lists are kept: fixed 64-byte messages; a transmit slot
// costs the sender one atomic fetch-and-increment; a message is sent with one store instruction
// (four lanes, 16 bytes each); flow control is off the critical path (the sender looks at the
// host's consumed count only when the ring could be full); completions are allocated
// independently of slots, so replies may come out of order; the GPU needs no progress thread; both
// directions use stores only (the host answers by storing a tag into a completion word the GPU
// polls).  One host thread serves the ring.
//
// Message layout (16 x uint32).  Every 16-byte quarter ends in the same generation tag, so the
// host accepts a message only when all four quarters of this generation have landed:
//   q0: op, calling PE, completion index (or NONE), tag
//   q1: dst address lo, hi, 0, tag      q2: src address lo, hi, 0, tag      q3: bytes lo, hi, 0, tag
// tag = 1 + (request index / ring slots), truncated to 32 bits, never 0.
#pragma once

#include <hsa/hsa.h>
#include <hsa/hsa_ext_amd.h>

#include <atomic>
#include <chrono>
#include <cstdint>
#include <cstring>
#include <memory>
#include <thread>
#include <vector>

enum : uint32_t { SHM_OFFLOAD_NOP = 0, SHM_OFFLOAD_COPY = 1, SHM_OFFLOAD_QUIET = 2 };
constexpr uint32_t SHM_OFFLOAD_NO_COMPLETION = 0xffffffffu;
constexpr uint32_t SHM_OFFLOAD_SLOTS = 4096;          // ring slots of 64 bytes (power of two)
constexpr uint32_t SHM_OFFLOAD_COMPLETIONS = 65536;   // completion words (power of two)

// Host-pinned block shared with the GPU.
struct shm_offload_shared {
    uint32_t ring[SHM_OFFLOAD_SLOTS][16];
    uint32_t completion[SHM_OFFLOAD_COMPLETIONS];
    uint64_t consumed;                // requests the host has taken out of the ring (flow control)
    uint64_t pad[7];
};

class shm_proxy {
public:
    // `shared` is zero-initialised pinned memory; agent/engines name the SDMA engines to use.
    void start(shm_offload_shared *shared, hsa_agent_t agent, const std::vector<uint32_t> &engines, int npes)
    {
        sh_ = shared;
        agent_ = agent;
        engines_ = engines;
        npes_ = static_cast<uint32_t>(npes);
        in_flight_per_pe_.reset(new std::atomic<uint32_t>[npes_]);
        for (uint32_t p = 0; p < npes_; ++p) in_flight_per_pe_[p].store(0);
        requests_in_flight_.clear();
        free_requests_.clear();
        stop_.store(false);
        stop_at_.store(0);
        taken_.store(0);
        requests_.store(0);
        copies_.store(0);
        failed_.store(0);
        thread_ = std::thread([this] { run(); });
    }

    // Ends the thread once it has taken every message up to ring index `head` (what the senders
    // have allocated so far) and the transfers it started have finished, both within a time limit.
    void stop(uint64_t head = 0)
    {
        if (!thread_.joinable()) return;
        stop_at_.store(head);
        stop_.store(true);
        thread_.join();
        for (hsa_signal_t s : free_) hsa_signal_destroy(s);
        free_.clear();
    }

    bool running() const { return thread_.joinable(); }
    uint64_t requests() const { return requests_.load(std::memory_order_relaxed); }
    uint64_t copies() const { return copies_.load(std::memory_order_relaxed); }

    // Requests whose engine transfer could not be started in full since the last call.
    uint64_t take_failed() { return failed_.exchange(0); }

    // The host side of quiet for transfers that kernels started through the ring: returns once the
    // thread has taken every message below ring index `head` and PE `pe` (every PE if pe < 0) has no
    // transfer in flight.  False if that has not happened after `limit_s` seconds.
    bool wait_idle(uint64_t head, int pe, double limit_s) const
    {
        const auto t0 = std::chrono::steady_clock::now();
        for (;;) {
            if (taken_.load(std::memory_order_acquire) >= head) {
                bool idle = true;
                for (uint32_t p = 0; p < npes_; ++p)
                    if ((pe < 0 || static_cast<uint32_t>(pe) == p) && in_flight_per_pe_[p].load(std::memory_order_acquire) != 0) idle = false;
                if (idle) return true;
            }
            if (std::chrono::duration<double>(std::chrono::steady_clock::now() - t0).count() > limit_s) return false;
            std::this_thread::yield();
        }
    }

private:
    // One request may be split into pieces that run on several engines; the requester is answered
    // when the last piece has finished.
    struct copy_in_flight {
        hsa_signal_t sig;
        uint32_t request;      // index into requests_in_flight_
    };
    struct request_in_flight {
        uint32_t pieces_left, pe, comp, tag;
    };
    struct quiet_waiting {
        uint32_t pe, comp, tag;
    };

    // Words that the other side (the GPU, or the CPU threads that play it in the host test)
    // writes or polls while this thread runs are touched with atomic accesses only: one aligned
    // load or store each (acquire and release cost nothing on the host), and a defined program
    // for a thread sanitizer.  A tag is read before the message it closes, and the consumed
    // count is published after the messages it covers have been copied out of their slots.
    static uint32_t peek(const uint32_t *word) { return __atomic_load_n(word, __ATOMIC_ACQUIRE); }
    void publish_consumed(uint64_t tail) { __atomic_store_n(&sh_->consumed, tail, __ATOMIC_RELEASE); }

    void reply(uint32_t comp, uint32_t tag)
    {
        if (comp == SHM_OFFLOAD_NO_COMPLETION) return;
        // one aligned 32-bit store; the GPU polls this word
        reinterpret_cast<std::atomic<uint32_t> *>(&sh_->completion[comp & (SHM_OFFLOAD_COMPLETIONS - 1)])->store(tag, std::memory_order_release);
    }

    bool take_signal(hsa_signal_t &s)
    {
        if (!free_.empty()) {
            s = free_.back();
            free_.pop_back();
        } else if (hsa_signal_create(1, 0, nullptr, &s) != HSA_STATUS_SUCCESS) {
            return false;
        }
        hsa_signal_store_relaxed(s, 1);
        return true;
    }

    void retire_copies()
    {
        for (size_t i = 0; i < copies_in_flight_.size();) {
            copy_in_flight &c = copies_in_flight_[i];
            if (hsa_signal_load_scacquire(c.sig) < 1) {
                request_in_flight &r = requests_in_flight_[c.request];
                if (--r.pieces_left == 0) {
                    reply(r.comp, r.tag);
                    in_flight_per_pe_[r.pe].fetch_sub(1, std::memory_order_release);
                    free_requests_.push_back(c.request);
                }
                free_.push_back(c.sig);
                copies_in_flight_[i] = copies_in_flight_.back();
                copies_in_flight_.pop_back();
            } else {
                ++i;
            }
        }
        for (size_t i = 0; i < quiets_.size();) {
            if (in_flight_per_pe_[quiets_[i].pe].load(std::memory_order_relaxed) == 0) {
                reply(quiets_[i].comp, quiets_[i].tag);
                quiets_[i] = quiets_.back();
                quiets_.pop_back();
            } else {
                ++i;
            }
        }
    }

    void handle(const uint32_t *m, uint32_t comp_tag)
    {
        const uint32_t op = m[0], pe = m[1], comp = m[2];
        requests_.fetch_add(1, std::memory_order_relaxed);
        if (pe >= npes_) {
            reply(comp, comp_tag);
            return;
        }
        if (op == SHM_OFFLOAD_COPY) {
            void *dst = reinterpret_cast<void *>(static_cast<uint64_t>(m[4]) | (static_cast<uint64_t>(m[5]) << 32));
            const void *src = reinterpret_cast<const void *>(static_cast<uint64_t>(m[8]) | (static_cast<uint64_t>(m[9]) << 32));
            const size_t n = static_cast<uint64_t>(m[12]) | (static_cast<uint64_t>(m[13]) << 32);
            if (n == 0 || engines_.empty()) {
                reply(comp, comp_tag);
                return;
            }
            // pieces of at least kMinPiece, 256-byte aligned, on successive engines
            size_t pieces = n / kMinPiece;
            if (pieces < 1) pieces = 1;
            if (pieces > engines_.size()) pieces = engines_.size();
            if (pieces > kMaxPieces) pieces = kMaxPieces;
            const size_t per = ((n + pieces - 1) / pieces + 255) & ~static_cast<size_t>(255);
            uint32_t request;
            if (!free_requests_.empty()) {
                request = free_requests_.back();
                free_requests_.pop_back();
            } else {
                request = static_cast<uint32_t>(requests_in_flight_.size());
                requests_in_flight_.push_back({});
            }
            uint32_t started = 0;
            for (size_t off = 0; off < n; off += per) {
                const size_t len = n - off < per ? n - off : per;
                hsa_signal_t sig;
                if (!take_signal(sig)) break;
                const uint32_t eng = engines_[next_engine_++ % engines_.size()];
                if (hsa_amd_memory_async_copy_on_engine(static_cast<char *>(dst) + off, agent_, static_cast<const char *>(src) + off, agent_,
                                                        len, 0, nullptr, sig, static_cast<hsa_amd_sdma_engine_id_t>(eng),
                                                        true) != HSA_STATUS_SUCCESS) {
                    free_.push_back(sig);
                    break;
                }
                copies_in_flight_.push_back({sig, request});
                ++started;
                copies_.fetch_add(1, std::memory_order_relaxed);
            }
            const bool all = static_cast<size_t>(started) * per >= n;
            if (!all) failed_.fetch_add(1);      // the requester is still released; the host's next quiet reports the failure
            if (started == 0) {
                free_requests_.push_back(request);
                reply(comp, comp_tag);
                return;
            }
            requests_in_flight_[request] = {started, pe, comp, comp_tag};
            in_flight_per_pe_[pe].fetch_add(1, std::memory_order_relaxed);
        } else if (op == SHM_OFFLOAD_QUIET) {
            if (in_flight_per_pe_[pe].load(std::memory_order_relaxed) == 0)
                reply(comp, comp_tag);
            else
                quiets_.push_back({pe, comp, comp_tag});
        } else {
            reply(comp, comp_tag);
        }
    }

    void run()
    {
        uint64_t tail = 0;
        uint32_t idle = 0;
        std::chrono::steady_clock::time_point stop_seen{};
        for (;;) {
            if (stop_.load(std::memory_order_acquire)) {
                // asked to end: first take what the senders had already put into the ring (bounded)
                const auto now = std::chrono::steady_clock::now();
                if (stop_seen == std::chrono::steady_clock::time_point{}) stop_seen = now;
                if (tail >= stop_at_.load(std::memory_order_relaxed) || std::chrono::duration<double>(now - stop_seen).count() > 5.0) break;
            }
            // Look at the next kBatch slots at once: their tag loads are independent, so the cache
            // misses (the GPU's stores evicted these lines from the host's caches) overlap instead of
            // being paid one message at a time.  Messages are taken strictly in ring order.
            bool complete[kBatch];
            for (unsigned i = 0; i < kBatch; ++i) {
                const uint64_t at = tail + i;
                const uint32_t *v = sh_->ring[at & (SHM_OFFLOAD_SLOTS - 1)];
                const uint32_t tag = static_cast<uint32_t>(at / SHM_OFFLOAD_SLOTS) + 1;
                complete[i] = peek(v + 3) == tag && peek(v + 7) == tag && peek(v + 11) == tag && peek(v + 15) == tag;
            }
            unsigned ready = 0;
            while (ready < kBatch && complete[ready]) ++ready;
            if (ready) {
                std::atomic_thread_fence(std::memory_order_acquire);
                for (unsigned i = 0; i < ready; ++i) {
                    uint32_t m[16];
                    memcpy(m, sh_->ring[tail & (SHM_OFFLOAD_SLOTS - 1)], sizeof m);
                    // completion tags count completion-word generations: 1 + (completion index / words)
                    handle(m, m[2] == SHM_OFFLOAD_NO_COMPLETION ? 0u : (m[2] / SHM_OFFLOAD_COMPLETIONS) + 1u);
                    ++tail;
                    if ((tail & 63) == 0) publish_consumed(tail);   // flow control, off the critical path
                }
                taken_.store(tail, std::memory_order_release);
                idle = 0;
            } else if (++idle == 64) {
                publish_consumed(tail);
                idle = 0;
            }
            if (!copies_in_flight_.empty() || !quiets_.empty()) retire_copies();
        }
        // leave nothing in flight
        const auto t0 = std::chrono::steady_clock::now();
        while (!copies_in_flight_.empty() && std::chrono::duration<double>(std::chrono::steady_clock::now() - t0).count() < 10.0)
            retire_copies();
    }

    shm_offload_shared *sh_ = nullptr;
    hsa_agent_t agent_{};
    std::vector<uint32_t> engines_;
    uint32_t npes_ = 0;
    std::unique_ptr<std::atomic<uint32_t>[]> in_flight_per_pe_;     // requests with unfinished pieces; read by wait_idle
    static constexpr unsigned kBatch = 8;              // ring slots examined per poll
    static constexpr size_t kMinPiece = 4u << 20;      // do not split below 4 MiB per engine
    static constexpr size_t kMaxPieces = 8;

    std::vector<copy_in_flight> copies_in_flight_;
    std::vector<request_in_flight> requests_in_flight_;
    std::vector<uint32_t> free_requests_;
    std::vector<quiet_waiting> quiets_;
    std::vector<hsa_signal_t> free_;
    std::atomic<bool> stop_{false};
    std::atomic<uint64_t> stop_at_{0};
    std::atomic<uint64_t> taken_{0};                   // ring messages handled so far
    std::thread thread_;
    std::atomic<uint64_t> requests_{0}, copies_{0}, failed_{0};
    uint32_t next_engine_ = 0;
};
