// The copy-engine transport: SDMA engines of the GPU, driven through the HSA runtime.
//
// On one device hipMemcpyAsync does not use the SDMA engines (the runtime runs a copy kernel
// instead), so the paper's "copy engine" path (section "Xe-Link Capabilities": engines that move
// data while the compute units stay free, at the price of a start-up latency) is reached with
// hsa_amd_memory_async_copy_on_engine, which can be forced onto an SDMA engine.  A transfer is
// asynchronous from submission until drain(): that is OpenSHMEM's non-blocking put, complete at
// quiet.  Host-only code; no kernels.
#pragma once

#include <hsa/hsa.h>
#include <hsa/hsa_ext_amd.h>

#include <chrono>
#include <cstddef>
#include <cstdint>
#include <string>
#include <vector>

class shm_copy_engines {
public:
    // Finds the HSA agent of the HIP device with PCI location (domain, bus, device) -- or, if no
    // agent reports that location, the `ordinal`-th GPU agent -- and lists its usable SDMA engines.
    bool init(int pci_domain, int pci_bus, int pci_device, int ordinal, int max_pes, std::string &err)
    {
        if (hsa_init() != HSA_STATUS_SUCCESS) {
            err = "hsa_init failed";
            return false;
        }
        inited_ = true;
        find_ctx f{pci_domain, pci_bus, pci_device, ordinal, 0, false, {}, false, {}, false, {}};
        hsa_iterate_agents(&shm_copy_engines::visit, &f);
        if (!f.match && !f.have_nth) {
            err = "no HSA GPU agent found";
            return false;
        }
        agent_ = f.match ? f.by_bdf : f.nth;
        // Engines usable for a copy that stays on this agent.  Older runtimes answer "none" for
        // that question although a forced engine copy works on every engine they list for
        // host<->device traffic; then that list is used, minus the two lowest engines, which the
        // HIP runtime itself keeps busy with host copies.
        uint32_t mask = 0;
        if (hsa_amd_memory_copy_engine_status(agent_, agent_, &mask) != HSA_STATUS_SUCCESS || mask == 0) {
            mask = 0;
            if (f.have_cpu) (void)hsa_amd_memory_copy_engine_status(agent_, f.cpu, &mask);
            if (mask & ~0x3u) mask &= ~0x3u;
        }
        if (mask == 0) {
            err = "the device reports no available SDMA engine";
            return false;
        }
        for (int b = 0; b < 16; ++b)
            if (mask & (1u << b)) engines_.push_back(1u << b);
        pending_.assign(max_pes, {});
        ready_ = true;
        return true;
    }

    bool ready() const { return ready_; }
    size_t n_engines() const { return engines_.size(); }
    hsa_agent_t agent() const { return agent_; }
    const std::vector<uint32_t> &engine_ids() const { return engines_; }

    // Start copying n bytes on behalf of PE `pe`.  Large transfers are cut into pieces of at least
    // kMinPiece bytes that run on several engines: as many as an equal share of the engines among
    // the PEs that have transfers in flight right now (this one included) allows, so that one PE
    // alone can use every engine and many PEs together still keep all of them busy.  Pieces go to
    // the engines round-robin over all transfers.
    bool submit(void *dst, const void *src, size_t n, int pe, int npes, std::string &err)
    {
        (void)npes;
        size_t active = 1;
        for (size_t p = 0; p < pending_.size(); ++p)
            if (static_cast<int>(p) != pe && !pending_[p].empty()) ++active;
        size_t share = (engines_.size() + active - 1) / active;
        if (share < 1) share = 1;
        size_t pieces = n / kMinPiece;
        if (pieces < 1) pieces = 1;
        if (pieces > share) pieces = share;
        const size_t per = ((n + pieces - 1) / pieces + 255) & ~static_cast<size_t>(255);
        for (size_t i = 0, off = 0; i < pieces && off < n; ++i, off += per) {
            const size_t len = (n - off < per) ? n - off : per;
            hsa_signal_t sig;
            if (!take_signal(sig)) {
                err = "hsa_signal_create failed";
                return false;
            }
            const uint32_t eng = engines_[next_engine_++ % engines_.size()];
            const hsa_status_t rc = hsa_amd_memory_async_copy_on_engine(
                static_cast<char *>(dst) + off, agent_, static_cast<const char *>(src) + off, agent_, len, 0, nullptr, sig,
                static_cast<hsa_amd_sdma_engine_id_t>(eng), true);
            if (rc != HSA_STATUS_SUCCESS) {
                const char *text = "";
                hsa_status_string(rc, &text);
                err = std::string("hsa_amd_memory_async_copy_on_engine: ") + text;
                free_.push_back(sig);
                return false;
            }
            pending_[pe].push_back(sig);
        }
        return true;
    }

    bool busy(int pe) const { return !pending_[pe].empty(); }

    // Wait for every transfer PE `pe` has started.  Bounded: a copy that has not finished after
    // `limit_s` seconds is reported instead of waited for; the transfers already retired leave the
    // pending list, the others stay on it (each signal is recycled exactly once).  A transfer the
    // engine ended with an error leaves its signal negative: it is retired and reported.
    bool drain(int pe, std::string &err, double limit_s = 60.0)
    {
        using clock = std::chrono::steady_clock;
        const auto t0 = clock::now();
        std::vector<hsa_signal_t> &q = pending_[pe];
        bool ok = true;
        size_t done = 0;
        for (; done < q.size(); ++done) {
            hsa_signal_value_t v;
            bool late = false;
            while ((v = hsa_signal_wait_scacquire(q[done], HSA_SIGNAL_CONDITION_LT, 1, 50000000ull, HSA_WAIT_STATE_ACTIVE)) >= 1) {
                if (std::chrono::duration<double>(clock::now() - t0).count() > limit_s) {
                    late = true;
                    break;
                }
            }
            if (late) {
                err = "a copy-engine transfer did not complete in time";
                ok = false;
                break;
            }
            if (v < 0) {
                err = "a copy-engine transfer ended with an error";
                ok = false;
            }
            free_.push_back(q[done]);
        }
        q.erase(q.begin(), q.begin() + static_cast<std::ptrdiff_t>(done));
        return ok;
    }

    void shutdown()
    {
        std::string ignore;
        for (size_t p = 0; p < pending_.size(); ++p) drain(static_cast<int>(p), ignore, 10.0);
        // a signal whose transfer never ended is leaked rather than destroyed under the engine
        for (hsa_signal_t s : free_) hsa_signal_destroy(s);
        free_.clear();
        if (inited_) hsa_shut_down();
        inited_ = ready_ = false;
    }

private:
    static constexpr size_t kMinPiece = 4u << 20;     // do not split below 4 MiB per engine

    struct find_ctx {
        int domain, bus, device, ordinal, seen;
        bool match;
        hsa_agent_t by_bdf;
        bool have_nth;
        hsa_agent_t nth;
        bool have_cpu;
        hsa_agent_t cpu;
    };

    static hsa_status_t visit(hsa_agent_t a, void *data)
    {
        find_ctx *f = static_cast<find_ctx *>(data);
        hsa_device_type_t type;
        if (hsa_agent_get_info(a, HSA_AGENT_INFO_DEVICE, &type) != HSA_STATUS_SUCCESS) return HSA_STATUS_SUCCESS;
        if (type == HSA_DEVICE_TYPE_CPU && !f->have_cpu) {
            f->cpu = a;
            f->have_cpu = true;
        }
        if (type != HSA_DEVICE_TYPE_GPU) return HSA_STATUS_SUCCESS;
        if (f->seen == f->ordinal) {
            f->nth = a;
            f->have_nth = true;
        }
        ++f->seen;
        uint32_t bdf = 0, domain = 0;
        if (hsa_agent_get_info(a, static_cast<hsa_agent_info_t>(HSA_AMD_AGENT_INFO_BDFID), &bdf) == HSA_STATUS_SUCCESS &&
            hsa_agent_get_info(a, static_cast<hsa_agent_info_t>(HSA_AMD_AGENT_INFO_DOMAIN), &domain) == HSA_STATUS_SUCCESS) {
            const int bus = (bdf >> 8) & 0xff, dev = (bdf >> 3) & 0x1f;
            if (!f->match && static_cast<int>(domain) == f->domain && bus == f->bus && dev == f->device) {
                f->by_bdf = a;
                f->match = true;
            }
        }
        return HSA_STATUS_SUCCESS;
    }

    bool take_signal(hsa_signal_t &sig)
    {
        if (!free_.empty()) {
            sig = free_.back();
            free_.pop_back();
        } else if (hsa_signal_create(1, 0, nullptr, &sig) != HSA_STATUS_SUCCESS) {
            return false;
        }
        hsa_signal_store_relaxed(sig, 1);
        return true;
    }

    bool inited_ = false, ready_ = false;
    size_t next_engine_ = 0;
    hsa_agent_t agent_{};
    std::vector<uint32_t> engines_;
    std::vector<hsa_signal_t> free_;
    std::vector<std::vector<hsa_signal_t>> pending_;
};
