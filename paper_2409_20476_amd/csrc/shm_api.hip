// C ABI of libshm355.so: context, symmetric heap, host-initiated operations, the cutover policy
// and the kernel-launch entry points.  Declarations and contracts are in include/shm355.h.
#include "shm355.h"

#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstdarg>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <mutex>
#include <new>
#include <string>

#include "shm_engine.hpp"
#include "shm_heap.hpp"
#include "shm_kernels.hpp"
#include "shm_proxy.hpp"

// Scratch memory of shm_launch_ring_pipeline_static, the entry point that allocates nothing: the
// arrival counters of the ring (one per chunk and PE) live here instead of in the heap's tail.  Every
// GPU the library runs on holds its own copy of the array until the process ends.  In host code the
// name is only a handle for hipGetSymbolAddress: the device address it yields, kept per device, is
// what kernels and clears are given.
static __device__ __align__(256) unsigned long long scratch[SHM_MAX_PES * SHM_STATIC_RING_MAX_CHUNKS];

namespace {

constexpr uint32_t ARRIVE_SLOTS = 4096;                       // 8-byte arrival counters per PE
static_assert(ARRIVE_SLOTS * 8 <= SHM_INTERNAL_BYTES, "arrival counters must fit the internal tail");
static_assert(SHM_WG_SIZE == SHMK_WG, "one work-group size everywhere");
constexpr int MAX_N_WG = 1 << 20;
// Group-owned tiles are the form for long messages moved by 64 or more groups (measured on MI355X,
// 32-256 MiB per PE).  A grid that fills the chip gains 5-10 % over the 8-group virtual blocks; eight
// PEs launching 64 groups each on their own streams gain 6-9 points of the HBM roofline (61 -> 67-70 %);
// one PE launching 64 groups ALONE loses 6 % (3.3 -> 3.1 TB/s of traffic) and 256 groups alone are
// level from 64 MiB -- the launcher cannot know who else is running and takes the case of all PEs at
// work, which is what the PEs of a context are for.  Fewer than 64 groups stay on the virtual blocks,
// which keep more loads in flight per group.
constexpr size_t TILES_MIN_BYTES = 32u << 20;
constexpr size_t TILE_BYTES = 64u << 10, TILES_PER_GROUP = 4;
constexpr long long TILES_MIN_GRID_GROUPS = 64;               // groups asked for, all PEs of the grid together
constexpr long long TILES_MIN_LAUNCHED_GROUPS = 64;           // groups launched, all PEs of the grid together
constexpr unsigned TILES_LDS_BYTES = 54000;                   // unused LDS that caps a CU at 3 resident groups
constexpr size_t TIMED_TICKET_GROUPS = 96;
constexpr size_t TIMED_TILES_MIN_BYTES = size_t(16) << 20;                    // groups per PE of a timed put whose tiles are dealt by ticket
constexpr uint64_t OFFLOAD_COUNTERS = 32768;                  // offset of the ring's three index words in PE 0's internal tail
static_assert(ARRIVE_SLOTS * 8 <= OFFLOAD_COUNTERS && OFFLOAD_COUNTERS + 24 <= SHMD_INTERNAL_SYNC_COUNT &&
                  SHMD_INTERNAL_SYNC_EPOCH + 8 <= SHMD_INTERNAL_QUIET && SHMD_INTERNAL_QUIET + 8 * 128 <= SHMD_INTERNAL_TICKETS &&
                  SHMD_INTERNAL_TICKETS + 8 * SHMD_TICKET_WORDS <= SHM_INTERNAL_BYTES,
              "internal tail layout");
static_assert(SHM_OFFLOAD_SLOTS == SHMD_OFFLOAD_SLOTS && SHM_OFFLOAD_COMPLETIONS == SHMD_OFFLOAD_COMPLETIONS &&
                  SHM_OFFLOAD_NO_COMPLETION == SHMD_OFFLOAD_NONE, "host and device agree on the ring");

thread_local std::string g_err = "";

constexpr int MAX_DEVICES = 64;
std::mutex g_scratch_mutex;
unsigned long long *g_scratch_ptr[MAX_DEVICES] = {};          // device address of `scratch` on each device, once asked for

int fail(int code, const char *fmt, ...)
{
    char buf[512];
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(buf, sizeof buf, fmt, ap);
    va_end(ap);
    g_err = buf;
    return code;
}

}  // namespace

struct shm_ctx {
    int npes = 0;
    size_t part_bytes = 0;        // partition stride = heap bytes per PE including the internal tail
    size_t user_bytes = 0;        // what callers may allocate and address
    char *base = nullptr;
    bool own_heap = false, own_streams = false, no_device = false;
    hipStream_t stream[SHM_MAX_PES] = {};
    hipEvent_t event[SHM_MAX_PES] = {};
    uint64_t *status_host = nullptr;
    uint64_t *status_dev = nullptr;
    uint64_t wait_us = 2000000;
    uint64_t ticks_per_us = 100;
    // AUTO thresholds per class of work-group count, as measured on MI355X with 8 PEs transferring at
    // once: the engines move more from 512 KiB with one group per PE and never against four or more
    // groups, given a hardware queue per PE stream; shm_init_ex lowers them when the process has
    // fewer hardware queues than PEs (default_cutovers).
    size_t cutover[4] = {size_t(512) << 10, SIZE_MAX, SIZE_MAX, SIZE_MAX};
    // AUTO thresholds of the collectives, bytes per PE, per class of work-group count; set at init
    // from the number of PEs (measured on MI355X with 4, 8 and 12 PEs; the host-started side of the
    // comparison is the runtime-copy path, which outruns the engines for these many-copy patterns).
    size_t coll_cutover[2][4] = {};
    bool team_sync = true;        // team launches order the PE streams (SHM_TEAM_SYNC_FULL or _TRACKED)
    bool team_tracked = false;    // ... but only those the library itself has used since the last team launch, and lazily
    bool pe_dirty[SHM_MAX_PES] = {};        // tracked mode: the library has enqueued work on this PE's stream since the last join
    bool pe_needs_fork[SHM_MAX_PES] = {};   // tracked mode: this PE's stream has not yet waited for the latest team work
    int num_cu = 0;
    uint32_t next_slot[SHM_MAX_PES] = {};
    shm_heap_allocator alloc;
    shm_copy_engines engines;     // SDMA engines through HSA; unused by a no-device context
    std::string engine_err;       // why the engines are unavailable, if they are
    shm_offload_shared *off_host = nullptr;   // pinned block of the reverse-offload ring
    shm_offload_shared *off_dev = nullptr;    // the same block at its device-visible address
    shm_proxy proxy;                          // host thread serving the ring
};

namespace {

#define HIP_TRY(expr)                                                                            \
    do {                                                                                         \
        hipError_t e_ = (expr);                                                                  \
        if (e_ != hipSuccess) return fail(SHM_EHIP, "%s: %s", #expr, hipGetErrorString(e_));     \
    } while (0)

shm_dev_ctx dev_view(const shm_ctx *c)
{
    shm_dev_ctx d;
    memset(&d, 0, sizeof d);
    for (int p = 0; p < c->npes; ++p) d.base[p] = c->base + static_cast<size_t>(p) * c->part_bytes;
    d.status = c->status_dev;
    d.wait_ticks = c->wait_us * c->ticks_per_us;
    d.stride = c->part_bytes;     // logical PEs are equal partitions of one allocation
    d.internal_off = c->user_bytes;
    d.npes = c->npes;
    if (c->off_dev && c->proxy.running()) {
        d.off.ring = &c->off_dev->ring[0][0];
        d.off.completion = &c->off_dev->completion[0];
        d.off.consumed = const_cast<const uint64_t *>(&c->off_dev->consumed);
        d.off.head = reinterpret_cast<unsigned long long *>(c->base + c->user_bytes + OFFLOAD_COUNTERS);
        d.off.comp_head = d.off.head + 1;
        d.off.consumed_seen = d.off.head + 2;
    }
    return d;
}

int check_ctx(const shm_ctx *c) { return c ? SHM_OK : fail(SHM_EINVAL, "null context"); }

int check_pe(const shm_ctx *c, int pe, const char *what)
{
    if (pe < 0 || pe >= c->npes) return fail(SHM_EPE, "%s %d outside 0..%d", what, pe, c->npes - 1);
    return SHM_OK;
}

int check_range(const shm_ctx *c, uint64_t off, size_t n, const char *what)
{
    if (off > c->user_bytes || n > c->user_bytes - off)
        return fail(SHM_ERANGE, "%s [%llu, +%zu) leaves the %zu-byte heap", what, (unsigned long long)off, n, c->user_bytes);
    return SHM_OK;
}

int check_word(const shm_ctx *c, uint64_t off, const char *what)
{
    if (int r = check_range(c, off, 8, what)) return r;
    if (off & 7) return fail(SHM_EINVAL, "%s offset %llu is not 8-byte aligned", what, (unsigned long long)off);
    return SHM_OK;
}

int check_n_wg(int n_wg)
{
    if (n_wg < 1 || n_wg > MAX_N_WG) return fail(SHM_EINVAL, "n_wg %d outside 1..%d", n_wg, MAX_N_WG);
    return SHM_OK;
}

// A team grid has n_wg x npes groups; a grid may not have 2^32 threads or more.
int check_team_grid(const shm_ctx *c, int n_wg)
{
    if (int r = check_n_wg(n_wg)) return r;
    if (static_cast<long long>(n_wg) * c->npes * SHMK_WG >= (1ll << 32))
        return fail(SHM_EINVAL, "%d groups for each of %d PEs exceed what one grid can hold (2^32 threads)", n_wg, c->npes);
    return SHM_OK;
}

bool overlaps(uint64_t a, uint64_t b, size_t n) { return n && a < b + n && b < a + n; }

int wg_class(int n_wg) { return n_wg <= 1 ? 0 : n_wg <= 4 ? 1 : n_wg <= 64 ? 2 : 3; }

int resolve_path(const shm_ctx *c, int path, size_t n, int n_wg, int *out)
{
    if (path == SHM_PATH_AUTO)      // a context without usable engines keeps to loads/stores
        *out = (n >= c->cutover[wg_class(n_wg)] && (c->no_device || c->engines.ready())) ? SHM_PATH_SDMA : SHM_PATH_LDST;
    else if (path == SHM_PATH_LDST || path == SHM_PATH_SDMA || path == SHM_PATH_MEMCPY)
        *out = path;
    else
        return fail(SHM_EINVAL, "unknown path %d", path);
    return SHM_OK;
}

// The HIP runtime gives a process GPU_MAX_HW_QUEUES hardware queues (4 unless the environment says
// otherwise) and spreads its streams over them.  With fewer queues than PEs the put kernels of
// different PEs' streams take turns, every per-PE load/store curve halves, and the engines --
// which are not in those queues -- win from smaller sizes: measured with 8 PEs on 4 queues, from
// 256 KiB against one group per PE and from 1-8 MiB (2 MiB taken) against four.
void default_cutovers(shm_ctx *c)
{
    int queues = 4;
    if (const char *e = getenv("GPU_MAX_HW_QUEUES")) {
        const int v = atoi(e);
        if (v >= 1) queues = v;
    }
    if (queues < c->npes) {
        c->cutover[0] = size_t(256) << 10;
        c->cutover[1] = size_t(2) << 20;
    }
}

void default_collective_cutovers(shm_ctx *c)
{
    const bool few = c->npes <= 4;
    const size_t fc[4] = {few ? size_t(512) << 10 : size_t(2) << 20, few ? size_t(2) << 20 : size_t(8) << 20, SIZE_MAX, SIZE_MAX};
    const size_t bc[4] = {size_t(256) << 10, size_t(1) << 20, size_t(16) << 20, SIZE_MAX};
    for (int k = 0; k < 4; ++k) {
        c->coll_cutover[SHM_COLL_FCOLLECT][k] = fc[k];
        c->coll_cutover[SHM_COLL_BROADCAST][k] = bc[k];
    }
}

int check_collective(int collective)
{
    if (collective != SHM_COLL_FCOLLECT && collective != SHM_COLL_BROADCAST) return fail(SHM_EINVAL, "unknown collective %d", collective);
    return SHM_OK;
}

// AUTO for a collective: the push kernel below the collective's own threshold, runtime copies from it on.
int resolve_collective_path(const shm_ctx *c, int collective, int path, size_t bytes_per_pe, int n_wg, int *out)
{
    if (path != SHM_PATH_AUTO) return resolve_path(c, path, bytes_per_pe, n_wg, out);
    *out = bytes_per_pe >= c->coll_cutover[collective][wg_class(n_wg)] ? SHM_PATH_MEMCPY : SHM_PATH_LDST;
    return SHM_OK;
}

int launched(const char *what)
{
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fail(SHM_EHIP, "launch of %s: %s", what, hipGetErrorString(e));
    return SHM_OK;
}

int no_device(const char *what) { return fail(SHM_ENODEV, "%s needs a device; context was built with SHM_INIT_NO_DEVICE", what); }

int take_status(shm_ctx *c)
{
    if (c->status_host && *c->status_host) {
        *c->status_host = 0;
        return fail(SHM_ETIMEOUT, "a device-side wait expired after %llu us", (unsigned long long)c->wait_us);
    }
    return SHM_OK;
}

// Ring index the senders have allocated up to now (the word lives in device memory).
int offload_head(const shm_ctx *c, uint64_t *head)
{
    *head = 0;
    if (!c->proxy.running()) return SHM_OK;
    HIP_TRY(hipMemcpy(head, c->base + c->user_bytes + OFFLOAD_COUNTERS, 8, hipMemcpyDeviceToHost));
    return SHM_OK;
}

// Host side of quiet for the engine transfers that kernels of PE `pe` (all PEs if pe < 0) started
// through the ring and did not wait for themselves.  The PE's stream must be idle already, so that
// every request of its kernels is in the ring.
int quiet_offloaded(shm_ctx *c, int pe)
{
    if (!c->proxy.running()) return SHM_OK;
    uint64_t head = 0;
    if (int r = offload_head(c, &head)) return r;
    if (!c->proxy.wait_idle(head, pe, 60.0)) return fail(SHM_ETIMEOUT, "engine transfers started by kernels did not complete in time");
    if (c->proxy.take_failed()) return fail(SHM_EHIP, "the host proxy could not start an engine transfer a kernel asked for");
    return SHM_OK;
}

// All PE streams -> team stream (PE 0's).
int team_join(shm_ctx *c)
{
    for (int p = 1; p < c->npes; ++p) {
        if (c->team_tracked && !c->pe_dirty[p]) continue;      // nothing of the library's on that stream since the last join
        HIP_TRY(hipEventRecord(c->event[p], c->stream[p]));
        HIP_TRY(hipStreamWaitEvent(c->stream[0], c->event[p], 0));
        c->pe_dirty[p] = false;
    }
    return SHM_OK;
}

// Team stream -> all PE streams.
int team_fork(shm_ctx *c)
{
    HIP_TRY(hipEventRecord(c->event[0], c->stream[0]));
    for (int p = 1; p < c->npes; ++p) {
        if (c->team_tracked)
            c->pe_needs_fork[p] = true;         // the wait is enqueued when that PE's stream is next used
        else
            HIP_TRY(hipStreamWaitEvent(c->stream[p], c->event[0], 0));
    }
    return SHM_OK;
}

// Tracked mode: PE pe's stream catches up with the team stream before it is used again.
int lazy_fork(shm_ctx *c, int pe)
{
    if (c->team_tracked && c->pe_needs_fork[pe]) {
        HIP_TRY(hipStreamWaitEvent(c->stream[pe], c->event[0], 0));
        c->pe_needs_fork[pe] = false;
    }
    return SHM_OK;
}

uint32_t take_slots(shm_ctx *c, int pe, uint32_t count)
{
    if (c->next_slot[pe] + count > ARRIVE_SLOTS) c->next_slot[pe] = 0;
    const uint32_t s = c->next_slot[pe];
    c->next_slot[pe] += count;
    return s;
}

int rma_args(const shm_ctx *c, int me, int pe, uint64_t dst_off, uint64_t src_off, size_t n)
{
    if (int r = check_pe(c, me, "calling PE")) return r;
    if (int r = check_pe(c, pe, "target PE")) return r;
    if (int r = check_range(c, dst_off, n, "destination")) return r;
    if (int r = check_range(c, src_off, n, "source")) return r;
    if (me == pe && overlaps(dst_off, src_off, n)) return fail(SHM_EINVAL, "source and destination overlap on PE %d", me);
    return SHM_OK;
}

// Wait for the copy-engine transfers PE `pe` has in flight, so that whatever is enqueued next on
// its stream finds them done.
int drain_engines(shm_ctx *c, int pe)
{
    if (!c->engines.ready() || !c->engines.busy(pe)) return SHM_OK;
    std::string err;
    if (!c->engines.drain(pe, err)) return fail(SHM_EHIP, "%s", err.c_str());
    return SHM_OK;
}

// Every launch on one PE's own stream starts here: that PE's engine transfers are finished (they are
// not on the stream) and, in tracked mode, the stream first catches up with the team stream and is
// marked as used.
int begin_pe_launch(shm_ctx *c, int pe)
{
    if (int r = drain_engines(c, pe)) return r;
    if (int r = lazy_fork(c, pe)) return r;
    c->pe_dirty[pe] = true;
    return SHM_OK;
}

int drain_all_engines(shm_ctx *c)
{
    for (int p = 0; p < c->npes; ++p)
        if (int r = drain_engines(c, p)) return r;
    return SHM_OK;
}

// What a team launch with nothing to move still owes its callers: with team sync on, everything
// enqueued before it on any PE stream is ordered before everything enqueued after it.
int team_order_only(shm_ctx *c)
{
    if (int r = drain_all_engines(c)) return r;      // engine transfers are not on the streams
    if (!c->team_sync) return SHM_OK;
    if (int r = team_join(c)) return r;
    return team_fork(c);
}


// Runtime copy: hipMemcpyAsync in stream order on PE `on_pe`'s stream.
int memcpy_copy(shm_ctx *c, int on_pe, int dst_pe, uint64_t dst_off, int src_pe, uint64_t src_off, size_t n)
{
    if (n == 0) return SHM_OK;
    if (int r = begin_pe_launch(c, on_pe)) return r;
    HIP_TRY(hipMemcpyAsync(shm_ptr(c, dst_off, dst_pe), shm_ptr(c, src_off, src_pe), n, hipMemcpyDeviceToDevice, c->stream[on_pe]));
    return SHM_OK;
}

// Copy engine: the host waits until PE `on_pe`'s stream is idle (the engines are not part of the
// stream), then starts the SDMA transfer; it runs asynchronously until that PE's quiet.
int sdma_copy(shm_ctx *c, int on_pe, int dst_pe, uint64_t dst_off, int src_pe, uint64_t src_off, size_t n)
{
    if (!c->engines.ready()) return fail(SHM_EHIP, "copy engines unavailable: %s", c->engine_err.c_str());
    if (n == 0) return SHM_OK;
    if (int r = lazy_fork(c, on_pe)) return r;
    HIP_TRY(hipStreamSynchronize(c->stream[on_pe]));
    std::string err;
    if (!c->engines.submit(shm_ptr(c, dst_off, dst_pe), shm_ptr(c, src_off, src_pe), n, on_pe, c->npes, err))
        return fail(SHM_EHIP, "%s", err.c_str());
    return SHM_OK;
}

// Groups per PE that the tile kernel is launched with for a request of n_wg groups.  Which bytes a
// group moves cannot be observed, so the launcher runs as many groups as give each of them four
// 64 KiB tiles (never more than it was asked for): measured on MI355X over 8 PEs x 64-256 MiB and ten
// placements of the buffers, four tiles per group is where the tile copy is both fastest on
// average and least dependent on the placement; with one tile per group (1024 groups per PE at
// 64 MiB) a group spends a tenth of its life starting up (78.5 % of the HBM roofline against 81 %),
// with eight or more the rate falls by about a point.
unsigned tile_groups(size_t n, int n_wg, size_t tiles_per_group = TILES_PER_GROUP)
{
    const size_t tiles = (n + TILE_BYTES - 1) / TILE_BYTES, want = (tiles + tiles_per_group - 1) / tiles_per_group;
    return static_cast<unsigned>(want < static_cast<size_t>(n_wg) ? (want ? want : 1) : n_wg);
}

// Team puts and gets of 32 MiB or more per PE asked of about 128 or more groups per PE (ticket_groups; from
// 128 MiB also of fewer: team_ticket_groups), in grids of two PEs or more, run that many groups per PE that stay in the kernel and draw half-tile pieces (32 KiB) by
// ticket, in address order, from a counter pair in their PE's tail (shm_copy_tiles_ticketed; the
// pair sets itself back, so a recorded launch replays).  Measured on MI355X over twelve random
// placements of the buffers, min / mean / max percent of the HBM roofline: 8 PEs x 256 MiB 83.9 /
// 84.1 / 84.4, 128 MiB 83.4 / 83.7 / 83.9, 64 MiB 82.2 / 82.6 / 83.0, 48 MiB 81.1 / 81.9 / 82.2, 32 MiB
// 79.5 / 80.4 / 80.9; 6 PEs x 256 / 64 MiB 84.2 / 82.0 mean; 4 PEs 83.7 / 80.6.  The forms it replaces:
// fronts (512 groups sweeping each 32 MiB segment together, 4 KiB per group and step) 77.4 / 79.2 / 80.1
// at 8 x 256 MiB and 74.8 / 79.9 / 81.7 at 64 MiB -- their rate follows the distance between destination
// and source modulo 128 MiB --, group-owned tiles 77-79 %.  The number of groups is the window: 128 x
// 32 KiB = 4 MiB per PE is what this memory system likes (112 or 144 groups: 81.6 % at 8 x 256 MiB, 96 or
// 192: 81.5, 256: 82.0; the same at 4 and 6 PEs).  Below 32 MiB per PE the virtual blocks stay: on buffers that
// nothing has touched for a while the two forms are level (8 PEs x 8 / 16 / 24 MiB: 25.4 / 45.6 / 66.6 us against 24.8 /
// 44.2 / 63.1 us by ticket), on buffers that sit in the 256 MiB memory-side cache the virtual blocks, which store such
// sizes write-through, are a quarter faster (18.8 / 33.8 / 48.4 us against 23.6 / 43.5 / 62.4 us).
constexpr size_t TICKETS_MIN_BYTES = size_t(32) << 20, FCOLLECT_TICKETS_MIN_BYTES = size_t(8) << 20, BROADCAST_TICKETS_MIN_BYTES = size_t(32) << 20;
constexpr int TICKET_GROUPS = 128, PER_PE_TICKET_MIN_GROUPS = 32, PER_PE_TICKET_MAX_GROUPS = 100;
constexpr size_t PER_PE_WAYS_MIN_BYTES = size_t(128) << 20;
static_assert(SHMD_INTERNAL_WAY_TICKETS >= SHMD_INTERNAL_TICKETS + 8 * SHMD_TICKET_WORDS &&
                  SHMD_INTERNAL_WAY_TICKETS + SHMD_TICKET_MAX_WAYS * SHMD_TICKET_WAY_BYTES <= SHM_INTERNAL_BYTES,
              "the pairs of walks in ways lie behind the ticket words, inside the internal tail");
// Groups per PE of a team launch by ticket: the whole grid is a multiple of the number of compute
// units (half a group per unit and PE, rounded down to whole groups per unit), 128 per PE on 256 units
// when the number of PEs is even.  With 128 per PE at an odd number of PEs some units hold one group
// more than others and the rate falls below the tiles' (3 PEs x 128 MiB 77.0 % against 78.9 %); 85
// groups per PE give 82.9 %, 170 give 79.4 %; 5 PEs: 102 groups 81.0 %, 128 78.5 %, 153 79.8 %, tiles 78.7 %;
// 7 PEs: 109 groups 81.2 %, 128 80.5 %, 73 79.8 %, tiles 78.5 %.  Even grids at 128 per PE: 2 PEs x 256 MiB
// 84.4 % (tiles 81.0 %), 10 / 12 / 16 PEs x 128 MiB 83.2 / 83.3 / 83.6 % (tiles 78.4-78.6 %); odd grids by this
// rule: 3 PEs x 256 MiB 84.9 %, 9 / 11 / 13 / 15 PEs x 128 MiB 81.1 / 81.4 / 81.6 / 81.9 % (tiles 78.4-78.7 %).
unsigned ticket_groups(const shm_ctx *c, int grid_pes)
{
    const int cus = c->num_cu > 0 ? c->num_cu : 2 * TICKET_GROUPS, rounds = std::max(1, grid_pes / 2);
    return static_cast<unsigned>(std::max(1, cus * rounds / grid_pes));
}
// The largest number of groups per PE, not above `groups`, that makes a team grid a whole number of
// groups per compute unit (`groups` itself when the grid has fewer groups than the chip has units).
// A grid that leaves some units with one group more than others runs at the pace of those units: team
// puts of 128 MiB per PE on group-owned tiles, % of the HBM roofline as asked -> rounded down: 8 PEs x 40 / 48 /
// 70 / 100 groups 65.5 / 73.7 / 70.0 / 72.3 -> 79.9 / 79.9 / 79.2 / 78.5; 4 PEs x 70 / 100 / 127: 60.9 / 76.4 / 78.1 ->
// 80.5 / 80.7 / 80.6; 6 PEs x 48 / 64 / 100: 61.4 / 75.0 / 73.2 -> 78.8 / 78.9 / 78.4; 3 PEs x 100 / 120 / 127: 62.9 / 70.7 /
// 72.8 -> 78.2 / 78.3 / 78.3; never slower in any case measured.
unsigned balanced_groups(const shm_ctx *c, unsigned groups, int grid_pes)
{
    const unsigned cus = c->num_cu > 0 ? static_cast<unsigned>(c->num_cu) : 256u;
    const unsigned per_cu = groups * static_cast<unsigned>(grid_pes) / cus;
    return per_cu == 0 ? groups : per_cu * cus / static_cast<unsigned>(grid_pes);
}
// Groups per PE with which a team put or get of n bytes per PE asked of n_wg groups per PE runs by ticket,
// or 0 if it does not (any byte addresses: the kernel walks from the destination's next 1 KiB boundary).
// From 32 MiB and ticket_groups() asked for: that many.  From 128 MiB also with fewer, as long as there is a
// group per compute unit in all: the largest whole number of groups per unit not above what was asked (%
// of the HBM roofline on balanced tiles -> by ticket, 256 / 128 MiB per PE: 8 PEs x 40-127 groups 77-79 -> 81.2,
// 78-80 -> 80.3-81.4; 4 PEs x 64-127 groups 79.5 -> 84.0, 79.3 -> 82.5; 6 PEs x 64-127 groups 78 -> 82-83, 78.5 -> 81-82.6;
// at 64 MiB the two are level or the tiles ahead).
// The team form keeps one pair per PE: walked in two ways (as a PE's own long launches are) grids of 2 / 3 / 4 PEs x
// 256 MiB measure 82.9 / 81.7 / 81.1 % against 84.2 / 84.6 / 83.5 %, and less at every smaller size.
constexpr size_t TICKETS_FEW_GROUPS_MIN_BYTES = size_t(128) << 20;
unsigned team_ticket_groups(const shm_ctx *c, size_t n, int n_wg)
{
    if (n < TICKETS_MIN_BYTES || c->npes < 2) return 0;
    const unsigned full = ticket_groups(c, c->npes);
    if (static_cast<unsigned>(n_wg) >= full) return full;
    if (n >= TICKETS_FEW_GROUPS_MIN_BYTES && static_cast<long long>(n_wg) * c->npes >= std::max(1, c->num_cu))
        return balanced_groups(c, static_cast<unsigned>(n_wg), c->npes);
    return 0;
}
// A PE's own launches asked of more than 100 groups stay on group-owned tiles below 128 MiB: eight per-PE kernels of 128 groups drawing tickets
// measure what the tiles do (78 % at 8 x 256 MiB, 75-77 % at 64-128 MiB) and one PE launching alone
// loses a quarter (4.9 against 6.5 TB/s of traffic); with 256 groups per kernel eight kernels gain 2.6 points
// at 256 MiB (80.9 %) and one alone falls from 81 to 60-64 %.  The launcher cannot know who else is running.
uint64_t ticket_pair_off(const shm_ctx *c, unsigned pair) { return c->user_bytes + SHMD_INTERNAL_TICKETS + 8ull * pair; }

// Long, 16-byte-aligned messages moved by a grid that fills the chip take the group-owned-tile kernel.
bool use_tiles(uint64_t dst_off, uint64_t src_off, size_t n, int n_wg, int grid_pes)
{
    return ((dst_off | src_off) & 15) == 0 && n >= TILES_MIN_BYTES && static_cast<long long>(n_wg) * grid_pes >= TILES_MIN_GRID_GROUPS &&
           static_cast<long long>(tile_groups(n, n_wg)) * grid_pes >= TILES_MIN_LAUNCHED_GROUPS;
}

int transfer_copy(shm_ctx *c, int path, int on_pe, int dst_pe, uint64_t dst_off, int src_pe, uint64_t src_off, size_t n)
{
    return path == SHM_PATH_SDMA ? sdma_copy(c, on_pe, dst_pe, dst_off, src_pe, src_off, n)
                                 : memcpy_copy(c, on_pe, dst_pe, dst_off, src_pe, src_off, n);
}

int wg_rma(shm_ctx *c, int me, int pe, uint64_t dst_off, uint64_t src_off, size_t n, int n_wg, int path, int is_get)
{
    if (int r = check_ctx(c)) return r;
    if (int r = rma_args(c, me, pe, dst_off, src_off, n)) return r;
    if (int r = check_n_wg(n_wg)) return r;
    int use;
    if (int r = resolve_path(c, path, n, n_wg, &use)) return r;
    if (c->no_device) return no_device(is_get ? "shm_launch_wg_get" : "shm_launch_wg_put");
    if (use != SHM_PATH_LDST)
        return is_get ? transfer_copy(c, use, me, me, dst_off, pe, src_off, n) : transfer_copy(c, use, me, pe, dst_off, me, src_off, n);
    if (int r = begin_pe_launch(c, me)) return r;
    const int shift = (pe - me + c->npes) % c->npes;
    // A PE's own long put or get asked of 32-100 groups runs exactly those groups by ticket (any byte addresses;
    // the PE's own counter pair): measured with 64 groups, 256 / 64 MiB, % of the HBM roofline, tiles -> tickets:
    // eight PEs launching at once 67.9 -> 78.2 and 62.9 -> 70.4, one PE alone 38.5 -> 42.3 and 37.3 -> 39.6; 32 groups:
    // eight 41.8 -> 57.7, alone 24.4 -> 23.7; 100 groups: eight 75.2 -> 81.1, alone 54.9 -> 58.2.  With 128 groups one PE
    // alone loses 4-5 points by ticket and with 192 or more 16 (one counter's window is too small for the whole
    // chip), so those stay on tiles: the launcher cannot know who else is running.
    if (n >= TICKETS_MIN_BYTES && n_wg >= PER_PE_TICKET_MIN_GROUPS && n_wg <= PER_PE_TICKET_MAX_GROUPS) {
        hipLaunchKernelGGL(shmk_wg_rma_tiles, dim3(n_wg, 1), dim3(SHMK_WG), TILES_LDS_BYTES, c->stream[me], c->base,
                           static_cast<uint64_t>(c->part_bytes), dst_off, src_off, n, c->npes, me, shift, is_get,
                           ticket_pair_off(c, SHMD_TICKET_PE), 1u);
        return launched("work-group put/get (by ticket)");
    }
    // From 128 MiB, asked of a group per compute unit or more, it runs a group per unit by ticket in TWO ways: the
    // message in two halves, half of the groups and a counter pair each, the pairs 4 KiB apart.  One counter cannot
    // serve a whole chip's draws (the memory side performs the atomics on one line, and on neighbouring lines, one after
    // another: one PE alone with 256 groups on one pair 61 % of the HBM roofline, on two pairs in neighbouring lines 80.5 %,
    // 4 KiB apart 81.3-82.3 %, in four ways 78 %).  Measured, tiles -> two ways: 256 MiB one PE alone 79.4-81.2 -> 81.3, eight PEs
    // at once 76.6-77.9 -> 80.6; 128 MiB 78 -> 76.5 and 76.0 -> 78.6; at 64 MiB one PE alone loses 5 points, so tiles below 128 MiB.
    if (n >= PER_PE_WAYS_MIN_BYTES && n_wg >= c->num_cu && c->num_cu >= 2) {
        hipLaunchKernelGGL(shmk_wg_rma_tiles, dim3(c->num_cu & ~1, 1), dim3(SHMK_WG), TILES_LDS_BYTES, c->stream[me], c->base,
                           static_cast<uint64_t>(c->part_bytes), dst_off, src_off, n, c->npes, me, shift, is_get,
                           c->user_bytes + SHMD_INTERNAL_WAY_TICKETS, 2u);
        return launched("work-group put/get (by ticket, two ways)");
    }
    if (use_tiles(dst_off, src_off, n, n_wg, 1)) {
        hipLaunchKernelGGL(shmk_wg_rma_tiles, dim3(tile_groups(n, n_wg), 1), dim3(SHMK_WG), TILES_LDS_BYTES, c->stream[me], c->base,
                           static_cast<uint64_t>(c->part_bytes), dst_off, src_off, n, c->npes, me, shift, is_get, uint64_t(0), 1u);
        return launched("work-group put/get (tiles)");
    }
    hipLaunchKernelGGL(shmk_wg_rma, dim3(n_wg, 1), dim3(SHMK_WG), 0, c->stream[me], dev_view(c), dst_off, src_off, n, me, shift,
                       is_get);
    return launched("work-group put/get");
}

int wg_rma_all(shm_ctx *c, int pe_shift, uint64_t dst_off, uint64_t src_off, size_t n, int n_wg, int path, int is_get)
{
    if (int r = check_ctx(c)) return r;
    if (pe_shift < 0 || pe_shift >= c->npes) return fail(SHM_EPE, "pe_shift %d outside 0..%d", pe_shift, c->npes - 1);
    if (int r = rma_args(c, 0, pe_shift, dst_off, src_off, n)) return r;   // shift 0 = every PE targets itself
    if (int r = check_team_grid(c, n_wg)) return r;
    int use;
    if (int r = resolve_path(c, path, n, n_wg, &use)) return r;
    if (c->no_device) return no_device("team put/get");
    if (int r = drain_all_engines(c)) return r;
    if (use != SHM_PATH_LDST) {
        if (c->team_sync) {
            if (int r = team_join(c)) return r;
            if (int r = team_fork(c)) return r;
        }
        for (int p = 0; p < c->npes; ++p) {
            const int t = (p + pe_shift) % c->npes;
            if (int r = is_get ? transfer_copy(c, use, p, p, dst_off, t, src_off, n) : transfer_copy(c, use, p, t, dst_off, p, src_off, n))
                return r;
        }
        if (c->team_sync) {
            // the engines are not on the streams: only the host can put later work of OTHER PEs behind them
            if (use == SHM_PATH_SDMA)
                if (int r = drain_all_engines(c)) return r;
            if (int r = team_join(c)) return r;
            if (int r = team_fork(c)) return r;
        }
        return SHM_OK;
    }
    if (c->team_sync)
        if (int r = team_join(c)) return r;
    if (const unsigned tkg = team_ticket_groups(c, n, n_wg)) {
        hipLaunchKernelGGL(shmk_wg_rma_tiles, dim3(tkg, c->npes), dim3(SHMK_WG), TILES_LDS_BYTES, c->stream[0], c->base,
                           static_cast<uint64_t>(c->part_bytes), dst_off, src_off, n, c->npes, 0, pe_shift, is_get,
                           ticket_pair_off(c, SHMD_TICKET_TEAM), 1u);
    } else if (use_tiles(dst_off, src_off, n, n_wg, c->npes)) {
        hipLaunchKernelGGL(shmk_wg_rma_tiles, dim3(balanced_groups(c, tile_groups(n, n_wg), c->npes), c->npes), dim3(SHMK_WG), TILES_LDS_BYTES, c->stream[0], c->base,
                           static_cast<uint64_t>(c->part_bytes), dst_off, src_off, n, c->npes, 0, pe_shift, is_get, uint64_t(0), 1u);
    } else {
        // from 4 MiB per PE the grid is a whole number of groups per compute unit here too (8 PEs x 24 MiB asked of
        // 70 / 100 groups: 65 / 69 -> 76 / 73 % of the HBM roofline, 8 MiB of 40 / 70: 62 / 62 -> 68 / 70 %; at 2 MiB mixed)
        if (n >= (size_t(4) << 20)) n_wg = static_cast<int>(balanced_groups(c, static_cast<unsigned>(n_wg), c->npes));
        hipLaunchKernelGGL(shmk_wg_rma, dim3(n_wg, c->npes), dim3(SHMK_WG), 0, c->stream[0], dev_view(c), dst_off, src_off, n, 0,
                           pe_shift, is_get);
    }
    if (int r = launched("team put/get")) return r;
    if (c->team_sync)
        if (int r = team_fork(c)) return r;
    return SHM_OK;
}

}  // namespace

namespace {

typedef void (*reduce_kernel)(shm_dev_ctx, uint64_t, uint64_t, size_t, uint64_t);

// Groups per PE a split reduction over nvec 16-byte vectors is launched with, and the counter pair its
// groups draw from (0: none).  When a PE's slice is walked on group-owned tiles (the kernels' rule:
// SHMK_OWNED_MIN_TILES or more tiles of 64 KiB per PE) a group beyond the number of tiles has nothing
// to do, and launching it only delays the groups of the later PEs in the dispatch order (measured: 8 x
// 64 MiB, 1024 groups asked for, 128 tiles per PE: 0.22 ms with the idle groups, 0.185 ms without).
// Which group folds which vectors cannot be observed, so the launcher runs one group per two tiles,
// never more groups than it was asked for.  From 96 tiles per PE, asked of a group per compute unit
// or more, it runs exactly one group per compute unit in all, and they draw quarter tiles of their
// PE's slice by ticket (measured over twelve random placements of the buffers, mean % of the HBM
// roofline, fixed tiles -> tickets: 8 PEs x 48 / 64 / 96 / 128 MiB 70.4 -> 75.9, 74.2 -> 77.1, 73.6 -> 78.4,
// 73.0 -> 79.4, and the spread over placements falls from 70.4-76.8 to 76.4-77.4 at 64 MiB; 6 PEs x 64 /
// 128 MiB 65.8 -> 75.2, 69.2 -> 78.3; 12 PEs x 128 MiB 68.0 -> 77.4; 16 PEs x 128 MiB 70.6 -> 78.3; 4 PEs level;
// 8 PEs x 32 MiB, 64 tiles per PE, 74.3 -> 72.7, hence the 96; other numbers of groups at 8 x 64 MiB:
// 16 per PE 54 %, 24: 69.5, 40: 68.1, 48: 72.9, 64: 74.7, 96: 72.9; half tiles 76.4, eighths 76.7).
constexpr size_t SPLIT_REDUCE_TICKETS_MIN_TILES = 96;
int split_reduce_groups(const shm_ctx *c, size_t nvec, int n_wg, uint64_t *ticket_pair)
{
    const size_t tiles = shmk_split_share(nvec, c->npes) / 4096;
    *ticket_pair = 0;
    if (tiles < SHMK_OWNED_MIN_TILES) return n_wg;
    const int per_cu = c->num_cu / c->npes > 0 ? c->num_cu / c->npes : 1;
    if (tiles >= SPLIT_REDUCE_TICKETS_MIN_TILES && n_wg >= per_cu) {
        *ticket_pair = ticket_pair_off(c, SHMD_TICKET_COLL);
        return per_cu;
    }
    const size_t want = tiles / 2 < SHMK_OWNED_MIN_TILES ? SHMK_OWNED_MIN_TILES : tiles / 2;      // two tiles per group measure 1-3 points above one
    return static_cast<int>(balanced_groups(c, want < static_cast<size_t>(n_wg) ? static_cast<unsigned>(want) : static_cast<unsigned>(n_wg), c->npes));
}

// Groups per PE of a duplicate reduction over `bytes` per PE: from 4 MiB a whole number of groups per
// compute unit in all, and a multiple of 8 per PE, which the kernels' XCD-aware numbering needs (with
// another count the npes readers of a share are spread over the XCDs and every one of them fetches it
// from HBM).
int duplicate_reduce_groups(const shm_ctx *c, size_t bytes, int n_wg)
{
    if (bytes < (size_t(4) << 20) || n_wg < 8) return n_wg;
    const unsigned g = balanced_groups(c, static_cast<unsigned>(n_wg), c->npes) & ~7u;
    return g ? static_cast<int>(g) : (n_wg & ~7);
}

// Whether the groups of an fcollect (or collect) of blocks of `bytes` draw their pieces by ticket: from 8 MiB
// with six PEs or more, from 64 MiB with four or five (measured, 1024 groups asked, % of the HBM roofline, tiles ->
// tickets, blocks of 8 / 16 / 64 / 96 MiB: 7 PEs 69.1 / 67.2 / 76.5 / 76.7 -> 70.6 / 74.3 / 84.0 / 84.2; 6 PEs 67.9 / 67.7 / 71.9 /
// 75.3 -> 68.6 / 71.4 / 80.2 / 81.3; 4 PEs 66.4 / 68.7 / 74.8 / 70.0 -> 62.3 / 65.9 / 75.7 / 75.8; 3 PEs 62.3 / 66.0 / 73.3 / 71.0 ->
// 56.8 / 62.6 / 69.6 / 70.6; 2 PEs 60.6 / 66.7 / 67.5 / 68.2 -> 45.4 / 54.2 / 63.6 / 65.6).
bool fcollect_by_ticket(const shm_ctx *c, size_t bytes)
{
    return (c->npes >= 6 && bytes >= FCOLLECT_TICKETS_MIN_BYTES) || (c->npes >= 4 && bytes >= (size_t(64) << 20));
}

template <typename T, int OP>
reduce_kernel reduce_kernel_of(bool split)
{
    return split ? shmk_reduce<T, OP, true> : shmk_reduce<T, OP, false>;
}

template <typename T>
reduce_kernel reduce_kernel_for(int op, bool bitwise_ok, bool split)
{
    switch (op) {
    case SHM_OP_MIN: return reduce_kernel_of<T, SHMD_OP_MIN>(split);
    case SHM_OP_MAX: return reduce_kernel_of<T, SHMD_OP_MAX>(split);
    case SHM_OP_SUM: return reduce_kernel_of<T, SHMD_OP_SUM>(split);
    case SHM_OP_PROD: return reduce_kernel_of<T, SHMD_OP_PROD>(split);
    case SHM_OP_AND: return bitwise_ok ? reduce_kernel_of<T, SHMD_OP_AND>(split) : nullptr;
    case SHM_OP_OR: return bitwise_ok ? reduce_kernel_of<T, SHMD_OP_OR>(split) : nullptr;
    case SHM_OP_XOR: return bitwise_ok ? reduce_kernel_of<T, SHMD_OP_XOR>(split) : nullptr;
    default: return nullptr;
    }
}

// Signed and unsigned integers of one width share every kernel except min and max.
reduce_kernel pick_reduce(int dtype, int op, bool split, size_t *elem)
{
    const bool order = op == SHM_OP_MIN || op == SHM_OP_MAX;
    switch (dtype) {
    case SHM_INT8: *elem = 1; return order ? reduce_kernel_for<int8_t>(op, true, split) : reduce_kernel_for<uint8_t>(op, true, split);
    case SHM_UINT8: *elem = 1; return reduce_kernel_for<uint8_t>(op, true, split);
    case SHM_INT16: *elem = 2; return order ? reduce_kernel_for<int16_t>(op, true, split) : reduce_kernel_for<uint16_t>(op, true, split);
    case SHM_UINT16: *elem = 2; return reduce_kernel_for<uint16_t>(op, true, split);
    case SHM_INT32: *elem = 4; return order ? reduce_kernel_for<int32_t>(op, true, split) : reduce_kernel_for<uint32_t>(op, true, split);
    case SHM_UINT32: *elem = 4; return reduce_kernel_for<uint32_t>(op, true, split);
    case SHM_INT64: *elem = 8; return order ? reduce_kernel_for<int64_t>(op, true, split) : reduce_kernel_for<uint64_t>(op, true, split);
    case SHM_UINT64: *elem = 8; return reduce_kernel_for<uint64_t>(op, true, split);
    case SHM_FLOAT32: *elem = 4; return reduce_kernel_for<float>(op, false, split);
    case SHM_FLOAT64: *elem = 8; return reduce_kernel_for<double>(op, false, split);
    default: *elem = 0; return nullptr;
    }
}

}  // namespace


extern "C" {

const char *shm_last_error(void) { return g_err.c_str(); }

int shm_init(int npes, size_t heap_bytes, void *heap_base, void *const *streams, shm_ctx **out)
{
    return shm_init_ex(npes, heap_bytes, heap_base, streams, SHM_INIT_DEFAULT, out);
}

int shm_init_ex(int npes, size_t heap_bytes, void *heap_base, void *const *streams, unsigned flags, shm_ctx **out)
{
    if (!out) return fail(SHM_EINVAL, "null out pointer");
    *out = nullptr;
    if (npes < 1 || npes > SHM_MAX_PES) return fail(SHM_EPE, "npes %d outside 1..%d", npes, SHM_MAX_PES);
    if (heap_bytes <= SHM_INTERNAL_BYTES || heap_bytes % 4096)
        return fail(SHM_EINVAL, "heap_bytes must be a multiple of 4096 larger than %d", SHM_INTERNAL_BYTES);
    if (heap_bytes > SIZE_MAX / SHM_MAX_PES) return fail(SHM_EINVAL, "heap_bytes too large");
    if (flags & ~static_cast<unsigned>(SHM_INIT_NO_DEVICE)) return fail(SHM_EINVAL, "unknown flags 0x%x", flags);
    if (reinterpret_cast<uintptr_t>(heap_base) & 255) return fail(SHM_EINVAL, "heap_base must be 256-byte aligned");
    shm_ctx *c = new (std::nothrow) shm_ctx;
    if (!c) return fail(SHM_ENOMEM, "out of host memory");
    c->npes = npes;
    c->part_bytes = heap_bytes;
    c->user_bytes = heap_bytes - SHM_INTERNAL_BYTES;
    c->alloc.reset(c->user_bytes);
    default_cutovers(c);
    default_collective_cutovers(c);
    c->no_device = (flags & SHM_INIT_NO_DEVICE) != 0;
    if (c->no_device) {
        if (!heap_base) {
            delete c;
            return fail(SHM_EINVAL, "SHM_INIT_NO_DEVICE needs a non-null heap_base placeholder");
        }
        c->base = static_cast<char *>(heap_base);
        *out = c;
        return SHM_OK;
    }
    auto bail = [&](int code) {
        shm_finalize(c);
        return code;
    };
#define INIT_TRY(expr)                                                                                   \
    do {                                                                                                 \
        hipError_t e_ = (expr);                                                                          \
        if (e_ != hipSuccess) return bail(fail(SHM_EHIP, "%s: %s", #expr, hipGetErrorString(e_)));       \
    } while (0)
    int dev = 0, rate_khz = 0;
    INIT_TRY(hipGetDevice(&dev));
    INIT_TRY(hipDeviceGetAttribute(&c->num_cu, hipDeviceAttributeMultiprocessorCount, dev));
    if (hipDeviceGetAttribute(&rate_khz, hipDeviceAttributeWallClockRate, dev) == hipSuccess && rate_khz >= 1000)
        c->ticks_per_us = static_cast<uint64_t>(rate_khz) / 1000;
    if (heap_base) {
        c->base = static_cast<char *>(heap_base);
    } else {
        void *p = nullptr;
        hipError_t e = hipMalloc(&p, heap_bytes * npes);
        if (e != hipSuccess) return bail(fail(SHM_ENOMEM, "hipMalloc of %zu bytes: %s", heap_bytes * npes, hipGetErrorString(e)));
        c->base = static_cast<char *>(p);
        c->own_heap = true;
    }
    if (streams) {
        for (int p = 0; p < npes; ++p) c->stream[p] = static_cast<hipStream_t>(streams[p]);
    } else {
        c->own_streams = true;
        for (int p = 0; p < npes; ++p) INIT_TRY(hipStreamCreateWithFlags(&c->stream[p], hipStreamNonBlocking));
    }
    for (int p = 0; p < npes; ++p) INIT_TRY(hipEventCreateWithFlags(&c->event[p], hipEventDisableTiming));
    void *st = nullptr;
    INIT_TRY(hipHostMalloc(&st, 64, hipHostMallocMapped | hipHostMallocCoherent));
    c->status_host = static_cast<uint64_t *>(st);
    *c->status_host = 0;
    void *st_dev = nullptr;
    INIT_TRY(hipHostGetDevicePointer(&st_dev, st, 0));
    c->status_dev = static_cast<uint64_t *>(st_dev);
    for (int p = 0; p < npes; ++p)
        INIT_TRY(hipMemset(c->base + static_cast<size_t>(p) * heap_bytes + c->user_bytes, 0, SHM_INTERNAL_BYTES));
    INIT_TRY(hipDeviceSynchronize());
    {
        int dom = 0, bus = 0, slot = 0;
        (void)hipDeviceGetAttribute(&dom, hipDeviceAttributePciDomainId, dev);
        (void)hipDeviceGetAttribute(&bus, hipDeviceAttributePciBusId, dev);
        (void)hipDeviceGetAttribute(&slot, hipDeviceAttributePciDeviceId, dev);
        // a device without usable engines keeps working; only SHM_PATH_SDMA then reports an error
        (void)c->engines.init(dom, bus, slot, dev, SHM_MAX_PES, c->engine_err);
    }
#undef INIT_TRY
    *out = c;
    return SHM_OK;
}

int shm_finalize(shm_ctx *c)
{
    if (int r = check_ctx(c)) return r;
    if (!c->no_device) {
        for (int p = 0; p < c->npes; ++p)
            if (c->stream[p] || !c->own_streams) (void)hipStreamSynchronize(c->stream[p]);
        uint64_t head = 0;
        (void)offload_head(c, &head);
        c->proxy.stop(head);
        if (c->off_host) (void)hipHostFree(c->off_host);
        c->engines.shutdown();
        for (int p = 0; p < c->npes; ++p) {
            if (c->event[p]) (void)hipEventDestroy(c->event[p]);
            if (c->own_streams && c->stream[p]) (void)hipStreamDestroy(c->stream[p]);
        }
        if (c->status_host) (void)hipHostFree(c->status_host);
        if (c->own_heap && c->base) (void)hipFree(c->base);
    }
    delete c;
    return SHM_OK;
}

int shm_n_pes(const shm_ctx *c) { return c ? c->npes : fail(SHM_EINVAL, "null context"); }

size_t shm_heap_bytes(const shm_ctx *c) { return c ? c->user_bytes : 0; }

int shm_malloc(shm_ctx *c, size_t bytes, size_t align, uint64_t *off)
{
    if (int r = check_ctx(c)) return r;
    if (!off) return fail(SHM_EINVAL, "null offset pointer");
    if (align == 0) align = 256;
    if (align & (align - 1)) return fail(SHM_EINVAL, "alignment %zu is not a power of two", align);
    if (bytes == 0) {
        *off = SHM_NULL_OFF;
        return SHM_OK;
    }
    uint64_t o = shm_heap_allocator::NPOS;
    try {
        o = c->alloc.allocate(bytes, align);
    } catch (const std::bad_alloc &) {       // the allocator's own book-keeping; nothing crosses the C boundary
        return fail(SHM_ENOMEM, "out of host memory");
    }
    if (o == shm_heap_allocator::NPOS) return fail(SHM_ENOMEM, "no free extent of %zu bytes (align %zu) in the symmetric heap", bytes, align);
    *off = o;
    return SHM_OK;
}

int shm_calloc(shm_ctx *c, size_t bytes, size_t align, uint64_t *off)
{
    if (int r = shm_malloc(c, bytes, align, off)) return r;
    if (bytes == 0 || c->no_device) return SHM_OK;
    hipError_t e = hipSuccess;
    for (int p = 0; p < c->npes && e == hipSuccess; ++p) e = hipMemsetAsync(shm_ptr(c, *off, p), 0, bytes, c->stream[p]);
    for (int p = 0; p < c->npes && e == hipSuccess; ++p) e = hipStreamSynchronize(c->stream[p]);
    if (e != hipSuccess) {
        (void)c->alloc.release(*off);
        *off = SHM_NULL_OFF;
        return fail(SHM_EHIP, "clearing the block: %s", hipGetErrorString(e));
    }
    return SHM_OK;
}

int shm_free(shm_ctx *c, uint64_t off)
{
    if (int r = check_ctx(c)) return r;
    if (off == SHM_NULL_OFF) return SHM_OK;
    try {
        if (!c->alloc.release(off)) return fail(SHM_EINVAL, "offset %llu is not a live block", (unsigned long long)off);
    } catch (const std::bad_alloc &) {
        return fail(SHM_ENOMEM, "out of host memory");
    }
    return SHM_OK;
}

void *shm_ptr(const shm_ctx *c, uint64_t off, int pe)
{
    if (!c || pe < 0 || pe >= c->npes || off >= c->part_bytes) return nullptr;
    return c->base + static_cast<size_t>(pe) * c->part_bytes + off;
}

int shm_write(shm_ctx *c, int pe, uint64_t off, const void *host, size_t n)
{
    if (int r = check_ctx(c)) return r;
    if (int r = check_pe(c, pe, "PE")) return r;
    if (int r = check_range(c, off, n, "destination")) return r;
    if (n && !host) return fail(SHM_EINVAL, "null host buffer");
    if (c->no_device) return no_device("shm_write");
    if (n) HIP_TRY(hipMemcpy(shm_ptr(c, off, pe), host, n, hipMemcpyHostToDevice));
    return SHM_OK;
}

int shm_read(shm_ctx *c, int pe, uint64_t off, void *host, size_t n)
{
    if (int r = check_ctx(c)) return r;
    if (int r = check_pe(c, pe, "PE")) return r;
    if (int r = check_range(c, off, n, "source")) return r;
    if (n && !host) return fail(SHM_EINVAL, "null host buffer");
    if (c->no_device) return no_device("shm_read");
    if (n) HIP_TRY(hipMemcpy(host, shm_ptr(c, off, pe), n, hipMemcpyDeviceToHost));
    return SHM_OK;
}

int shm_putmem(shm_ctx *c, int me, uint64_t dst_off, uint64_t src_off, size_t n, int pe)
{
    if (int r = check_ctx(c)) return r;
    if (int r = rma_args(c, me, pe, dst_off, src_off, n)) return r;
    if (c->no_device) return no_device("shm_putmem");
    return memcpy_copy(c, me, pe, dst_off, me, src_off, n);
}

int shm_getmem(shm_ctx *c, int me, uint64_t dst_off, uint64_t src_off, size_t n, int pe)
{
    if (int r = check_ctx(c)) return r;
    if (int r = rma_args(c, me, pe, dst_off, src_off, n)) return r;
    if (c->no_device) return no_device("shm_getmem");
    return memcpy_copy(c, me, me, dst_off, pe, src_off, n);
}

int shm_quiet(shm_ctx *c, int me)
{
    if (int r = check_ctx(c)) return r;
    if (int r = check_pe(c, me, "calling PE")) return r;
    if (c->no_device) return no_device("shm_quiet");
    if (int r = lazy_fork(c, me)) return r;          // team work for this PE runs on the team stream: wait for it too
    HIP_TRY(hipStreamSynchronize(c->stream[me]));
    if (int r = drain_engines(c, me)) return r;
    if (int r = quiet_offloaded(c, me)) return r;
    return take_status(c);
}

int shm_fence(shm_ctx *c, int me)
{
    if (int r = check_ctx(c)) return r;
    if (int r = check_pe(c, me, "calling PE")) return r;
    if (c->no_device) return no_device("shm_fence");
    if (int r = drain_engines(c, me)) return r;     // engine transfers are not in the stream: finish them
    return take_status(c);                          // the stream itself executes in order
}

int shm_barrier_all(shm_ctx *c)
{
    if (int r = check_ctx(c)) return r;
    if (c->no_device) return no_device("shm_barrier_all");
    for (int p = 0; p < c->npes; ++p) HIP_TRY(hipStreamSynchronize(c->stream[p]));
    if (int r = drain_all_engines(c)) return r;
    if (int r = quiet_offloaded(c, -1)) return r;
    for (int p = 0; p < c->npes; ++p) c->pe_dirty[p] = c->pe_needs_fork[p] = false;      // every stream is idle: nothing left to order
    return take_status(c);
}

int shm_set_cutover(shm_ctx *c, int n_wg, size_t bytes)
{
    if (int r = check_ctx(c)) return r;
    if (int r = check_n_wg(n_wg)) return r;
    c->cutover[wg_class(n_wg)] = bytes;
    return SHM_OK;
}

int shm_get_cutover(const shm_ctx *c, int n_wg, size_t *bytes)
{
    if (int r = check_ctx(c)) return r;
    if (int r = check_n_wg(n_wg)) return r;
    if (!bytes) return fail(SHM_EINVAL, "null out pointer");
    *bytes = c->cutover[wg_class(n_wg)];
    return SHM_OK;
}

int shm_choose_path(const shm_ctx *c, size_t n, int n_wg, int *path)
{
    if (int r = check_ctx(c)) return r;
    if (int r = check_n_wg(n_wg)) return r;
    if (!path) return fail(SHM_EINVAL, "null out pointer");
    return resolve_path(c, SHM_PATH_AUTO, n, n_wg, path);
}

int shm_set_collective_cutover(shm_ctx *c, int collective, int n_wg, size_t bytes)
{
    if (int r = check_ctx(c)) return r;
    if (int r = check_collective(collective)) return r;
    if (int r = check_n_wg(n_wg)) return r;
    c->coll_cutover[collective][wg_class(n_wg)] = bytes;
    return SHM_OK;
}

int shm_get_collective_cutover(const shm_ctx *c, int collective, int n_wg, size_t *bytes)
{
    if (int r = check_ctx(c)) return r;
    if (int r = check_collective(collective)) return r;
    if (int r = check_n_wg(n_wg)) return r;
    if (!bytes) return fail(SHM_EINVAL, "null out pointer");
    *bytes = c->coll_cutover[collective][wg_class(n_wg)];
    return SHM_OK;
}

int shm_choose_collective_path(const shm_ctx *c, int collective, size_t bytes_per_pe, int n_wg, int *path)
{
    if (int r = check_ctx(c)) return r;
    if (int r = check_collective(collective)) return r;
    if (int r = check_n_wg(n_wg)) return r;
    if (!path) return fail(SHM_EINVAL, "null out pointer");
    return resolve_collective_path(c, collective, SHM_PATH_AUTO, bytes_per_pe, n_wg, path);
}

int shm_set_wait_timeout_us(shm_ctx *c, uint64_t us)
{
    if (int r = check_ctx(c)) return r;
    if (us == 0 || us > 600ull * 1000 * 1000) return fail(SHM_EINVAL, "timeout must be 1 us .. 600 s");
    c->wait_us = us;
    return SHM_OK;
}

int shm_set_team_sync(shm_ctx *c, int mode)
{
    if (int r = check_ctx(c)) return r;
    if (mode != SHM_TEAM_SYNC_OFF && mode != SHM_TEAM_SYNC_FULL && mode != SHM_TEAM_SYNC_TRACKED)
        return fail(SHM_EINVAL, "unknown team sync mode %d", mode);
    if (!c->no_device)
        for (int p = 1; p < c->npes; ++p)
            if (int r = lazy_fork(c, p)) return r;      // waits owed under the tracked mode are enqueued before it is left
    for (int p = 0; p < c->npes; ++p) c->pe_needs_fork[p] = false, c->pe_dirty[p] = (mode == SHM_TEAM_SYNC_TRACKED);
    c->team_sync = mode != SHM_TEAM_SYNC_OFF;
    c->team_tracked = mode == SHM_TEAM_SYNC_TRACKED;
    return SHM_OK;
}

size_t shm_device_context_bytes(void) { return sizeof(shm_dev_ctx); }

int shm_device_context(const shm_ctx *c, void *out, size_t out_bytes)
{
    if (int r = check_ctx(c)) return r;
    if (!out) return fail(SHM_EINVAL, "null out pointer");
    if (out_bytes != sizeof(shm_dev_ctx))
        return fail(SHM_EINVAL, "the device view has %zu bytes in this build, the caller expects %zu", sizeof(shm_dev_ctx), out_bytes);
    const shm_dev_ctx d = dev_view(c);
    memcpy(out, &d, sizeof d);
    return SHM_OK;
}

void *shm_stream(const shm_ctx *c, int pe)
{
    if (!c || c->no_device || pe < 0 || pe >= c->npes) return nullptr;
    return c->stream[pe];
}

int shm_stream_used(shm_ctx *c, int pe)
{
    if (int r = check_ctx(c)) return r;
    if (int r = check_pe(c, pe, "PE")) return r;
    if (c->no_device) return no_device("shm_stream_used");
    return begin_pe_launch(c, pe);
}

int shm_launch_wg_put(shm_ctx *c, int me, int pe, uint64_t dst_off, uint64_t src_off, size_t n, int n_wg, int path)
{
    return wg_rma(c, me, pe, dst_off, src_off, n, n_wg, path, 0);
}

int shm_launch_wg_get(shm_ctx *c, int me, int pe, uint64_t dst_off, uint64_t src_off, size_t n, int n_wg, int path)
{
    return wg_rma(c, me, pe, dst_off, src_off, n, n_wg, path, 1);
}

int shm_launch_wg_put_all(shm_ctx *c, int pe_shift, uint64_t dst_off, uint64_t src_off, size_t n, int n_wg, int path)
{
    return wg_rma_all(c, pe_shift, dst_off, src_off, n, n_wg, path, 0);
}

int shm_launch_wg_get_all(shm_ctx *c, int pe_shift, uint64_t dst_off, uint64_t src_off, size_t n, int n_wg, int path)
{
    return wg_rma_all(c, pe_shift, dst_off, src_off, n, n_wg, path, 1);
}

int shm_launch_wg_put_timed(shm_ctx *c, int me, int pe, uint64_t dst_off, uint64_t src_off, size_t n, int n_wg, int reps,
                            uint64_t *dev_ticks)
{
    if (int r = check_ctx(c)) return r;
    if (int r = rma_args(c, me, pe, dst_off, src_off, n)) return r;
    if (int r = check_n_wg(n_wg)) return r;
    if (reps < 1 || reps > (1 << 20)) return fail(SHM_EINVAL, "reps outside 1..2^20");
    if (!dev_ticks) return fail(SHM_EINVAL, "null tick buffer");
    if (c->no_device) return no_device("shm_launch_wg_put_timed");
    if (int r = begin_pe_launch(c, me)) return r;
    // pieces by ticket pay from 16 MiB here (put + quiet, 8 PEs: 16 MiB 50 -> 54 % of the roofline, 24 MiB 50 -> 62 %; 8 MiB 41 -> 35 %)
    const bool tiles = ((dst_off | src_off) & 15) == 0 && n >= TIMED_TILES_MIN_BYTES && n_wg >= TILES_MIN_GRID_GROUPS;
    // A put that its own quiet follows keeps its groups in the kernel anyway; from 16 MiB they draw
    // half-tile pieces by ticket (shm_copy_tiles_ticketed), one counter per repetition in the PE's own tail,
    // cleared here -- this entry point is not for graph capture.  More repetitions than there are
    // counters take fixed shares, eight tiles or more per group.
    const size_t n_tiles = (n + TILE_BYTES - 1) / TILE_BYTES;
    const bool tickets = tiles && reps <= static_cast<int>(SHMD_TICKET_TIMED_WORDS);
    const size_t per_group = tickets ? std::max(TILES_PER_GROUP, n_tiles / TIMED_TICKET_GROUPS) : std::max(2 * TILES_PER_GROUP, n_tiles / 128);
    if (tickets)
        HIP_TRY(hipMemsetAsync(c->base + static_cast<size_t>(me) * c->part_bytes + c->user_bytes + SHMD_INTERNAL_TICKETS, 0, 8u * reps,
                               c->stream[me]));
    unsigned long long *ticks = reinterpret_cast<unsigned long long *>(dev_ticks);
    const dim3 tile_grid(tile_groups(n, n_wg, per_group));
    if (tickets)
        hipLaunchKernelGGL(shmk_wg_put_timed<2>, tile_grid, dim3(SHMK_WG), TILES_LDS_BYTES, c->stream[me], dev_view(c), dst_off, src_off, n, me,
                           pe, reps, ticks);
    else if (tiles)
        hipLaunchKernelGGL(shmk_wg_put_timed<1>, tile_grid, dim3(SHMK_WG), TILES_LDS_BYTES, c->stream[me], dev_view(c), dst_off, src_off, n, me,
                           pe, reps, ticks);
    else
        hipLaunchKernelGGL(shmk_wg_put_timed<0>, dim3(n_wg), dim3(SHMK_WG), 0, c->stream[me], dev_view(c), dst_off, src_off, n, me, pe, reps,
                           ticks);
    return launched("timed work-group put");
}

int shm_launch_stream_probe(shm_ctx *c, int kind, uint64_t dst_off, uint64_t src_off, size_t n, int n_wg)
{
    if (int r = check_ctx(c)) return r;
    if (kind < SHM_PROBE_READ || kind > SHM_PROBE_WRITE_TICKETS) return fail(SHM_EINVAL, "unknown probe kind %d", kind);
    if (int r = rma_args(c, 0, c->npes > 1 ? 1 : 0, dst_off, src_off, n)) return r;
    if (n == 0 || n % 65536 || ((dst_off | src_off) & 15)) return fail(SHM_EINVAL, "the probe moves whole 64 KiB tiles at 16-byte aligned offsets");
    if (int r = check_team_grid(c, n_wg)) return r;
    if (c->no_device) return no_device("shm_launch_stream_probe");
    if (kind == SHM_PROBE_COPY) return wg_rma_all(c, c->npes > 1 ? 1 : 0, dst_off, src_off, n, n_wg, SHM_PATH_LDST, 0);
    if (int r = drain_all_engines(c)) return r;
    if (c->team_sync)
        if (int r = team_join(c)) return r;
    const int shift = c->npes > 1 ? 1 : 0;
    const bool tiles = kind == SHM_PROBE_READ || kind == SHM_PROBE_WRITE;
    const dim3 grid(tiles ? tile_groups(n, n_wg) : n_wg, c->npes), block(SHMK_WG);
    const uint64_t pair = ticket_pair_off(c, SHMD_TICKET_PROBE);
    auto launch = [&](auto kernel) {
        hipLaunchKernelGGL(kernel, grid, block, TILES_LDS_BYTES, c->stream[0], dev_view(c), dst_off, src_off, n, shift, 0x5eedf00du, pair);
    };
    switch (kind) {
    case SHM_PROBE_READ: launch(shmk_stream_probe<0, 0>); break;
    case SHM_PROBE_WRITE: launch(shmk_stream_probe<1, 0>); break;
    case SHM_PROBE_READ_FRONT: launch(shmk_stream_probe<0, 1>); break;
    case SHM_PROBE_WRITE_FRONT: launch(shmk_stream_probe<1, 1>); break;
    case SHM_PROBE_READ_TICKETS: launch(shmk_stream_probe<0, 2>); break;
    default: launch(shmk_stream_probe<1, 2>); break;
    }
    if (int r = launched("stream probe")) return r;
    if (c->team_sync)
        if (int r = team_fork(c)) return r;
    return SHM_OK;
}

int shm_proxy_start(shm_ctx *c)
{
    if (int r = check_ctx(c)) return r;
    if (c->no_device) return no_device("shm_proxy_start");
    if (c->proxy.running()) return SHM_OK;
    if (!c->engines.ready()) return fail(SHM_EHIP, "copy engines unavailable: %s", c->engine_err.c_str());
    for (int p = 0; p < c->npes; ++p) HIP_TRY(hipStreamSynchronize(c->stream[p]));
    if (!c->off_host) {
        void *h = nullptr, *d = nullptr;
        HIP_TRY(hipHostMalloc(&h, sizeof(shm_offload_shared), hipHostMallocMapped | hipHostMallocCoherent));
        c->off_host = static_cast<shm_offload_shared *>(h);
        HIP_TRY(hipHostGetDevicePointer(&d, h, 0));
        c->off_dev = static_cast<shm_offload_shared *>(d);
    }
    memset(c->off_host, 0, sizeof(shm_offload_shared));
    HIP_TRY(hipMemset(c->base + c->user_bytes + OFFLOAD_COUNTERS, 0, 24));
    HIP_TRY(hipDeviceSynchronize());
    c->proxy.start(c->off_host, c->engines.agent(), c->engines.engine_ids(), c->npes);
    return SHM_OK;
}

int shm_proxy_stop(shm_ctx *c)
{
    if (int r = check_ctx(c)) return r;
    if (c->no_device) return no_device("shm_proxy_stop");
    for (int p = 0; p < c->npes; ++p) HIP_TRY(hipStreamSynchronize(c->stream[p]));
    uint64_t head = 0;
    if (int r = offload_head(c, &head)) return r;
    c->proxy.stop(head);       // takes what is still in the ring and finishes the transfers first
    if (c->proxy.take_failed()) return fail(SHM_EHIP, "the host proxy could not start an engine transfer a kernel asked for");
    return take_status(c);
}

int shm_proxy_stats(const shm_ctx *c, uint64_t *requests, uint64_t *copies)
{
    if (int r = check_ctx(c)) return r;
    if (requests) *requests = c->proxy.requests();
    if (copies) *copies = c->proxy.copies();
    return SHM_OK;
}

int shm_launch_rma_device_initiated(shm_ctx *c, int me, int pe, uint64_t dst_off, uint64_t src_off, size_t n, int n_wg, int wg_size,
                                    int is_get, int mode, size_t cutover, size_t cover, uint64_t consume_off, int reps,
                                    uint64_t *dev_ticks)
{
    if (int r = check_ctx(c)) return r;
    if (int r = rma_args(c, me, pe, dst_off, src_off, n)) return r;
    if (n_wg < 1 || n_wg > 1024) return fail(SHM_EINVAL, "n_wg outside 1..1024");
    if (mode < 0 || mode > 5) return fail(SHM_EINVAL, "mode outside 0..5");
    if (wg_size < 1 || wg_size > 1024) return fail(SHM_EINVAL, "wg_size outside 1..1024");
    if (mode != 0 && wg_size % 64) return fail(SHM_EINVAL, "the copy-engine modes need whole waves: wg_size must be a multiple of 64");
    if (reps < 1 || reps > (1 << 20)) return fail(SHM_EINVAL, "reps outside 1..2^20");
    if (consume_off != SHM_NO_CONSUME) {
        if (!is_get) return fail(SHM_EINVAL, "only a get has a local destination to consume");
        if (mode == 5) return fail(SHM_EINVAL, "a get left to the host's quiet has nothing to consume inside the kernel");
        if (int r = check_range(c, consume_off, n, "consume buffer")) return r;
        if (overlaps(consume_off, dst_off, n) || (me == pe && overlaps(consume_off, src_off, n)))
            return fail(SHM_EINVAL, "the consume buffer overlaps the transfer");
    }
    if (c->no_device) return no_device("shm_launch_rma_device_initiated");
    if (mode != 0 && !c->proxy.running()) return fail(SHM_EINVAL, "the host proxy is not running (shm_proxy_start)");
    if (int r = begin_pe_launch(c, me)) return r;
    unsigned long long *ticks = reinterpret_cast<unsigned long long *>(dev_ticks);
    auto launch = [&](auto kernel) {
        hipLaunchKernelGGL(kernel, dim3(n_wg), dim3(wg_size), 0, c->stream[me], dev_view(c), dst_off, src_off, n, me, pe, cutover, cover,
                           consume_off, reps, ticks);
    };
    switch (mode * 2 + (is_get ? 1 : 0)) {
    case 0: launch(shmk_rma_device_initiated<0, false>); break;
    case 1: launch(shmk_rma_device_initiated<0, true>); break;
    case 2: launch(shmk_rma_device_initiated<1, false>); break;
    case 3: launch(shmk_rma_device_initiated<1, true>); break;
    case 4: launch(shmk_rma_device_initiated<2, false>); break;
    case 5: launch(shmk_rma_device_initiated<2, true>); break;
    case 6: launch(shmk_rma_device_initiated<3, false>); break;
    case 7: launch(shmk_rma_device_initiated<3, true>); break;
    case 8: launch(shmk_rma_device_initiated<4, false>); break;
    case 9: launch(shmk_rma_device_initiated<4, true>); break;
    case 10: launch(shmk_rma_device_initiated<5, false>); break;
    case 11: launch(shmk_rma_device_initiated<5, true>); break;
    default: return fail(SHM_EINVAL, "mode outside 0..5");
    }
    return launched("device-initiated transfer");
}

int shm_launch_put_device_initiated(shm_ctx *c, int me, int pe, uint64_t dst_off, uint64_t src_off, size_t n, int n_wg, int wg_size,
                                    int mode, size_t cutover, int reps, uint64_t *dev_ticks)
{
    if (mode < 0 || mode > 3) return fail(SHM_EINVAL, "mode outside 0..3");
    if (!dev_ticks) return fail(SHM_EINVAL, "null tick buffer");
    return shm_launch_rma_device_initiated(c, me, pe, dst_off, src_off, n, n_wg, wg_size, 0, mode, cutover, 0, SHM_NO_CONSUME, reps,
                                           dev_ticks);
}

int shm_launch_scalar_pg(shm_ctx *c, int me, int pe, uint64_t dst_off, uint64_t src_off, size_t nelems, int elem_bytes, int is_get,
                         int n_wg)
{
    if (int r = check_ctx(c)) return r;
    if (elem_bytes != 1 && elem_bytes != 2 && elem_bytes != 4 && elem_bytes != 8)
        return fail(SHM_EINVAL, "element size %d is not 1, 2, 4 or 8", elem_bytes);
    if (nelems > c->user_bytes / static_cast<size_t>(elem_bytes)) return fail(SHM_ERANGE, "the elements leave the heap");
    if (int r = rma_args(c, me, pe, dst_off, src_off, nelems * elem_bytes)) return r;
    if ((dst_off | src_off) % static_cast<uint64_t>(elem_bytes)) return fail(SHM_EINVAL, "scalar put/get needs element-aligned offsets");
    if (int r = check_n_wg(n_wg)) return r;
    if (c->no_device) return no_device("shm_launch_scalar_pg");
    if (int r = begin_pe_launch(c, me)) return r;
    if (nelems == 0) return SHM_OK;
    const dim3 grid(n_wg), block(SHMK_WG);
    const shm_dev_ctx d = dev_view(c);
    const int g = is_get ? 1 : 0;
    switch (elem_bytes) {
    case 1: hipLaunchKernelGGL(shmk_scalar_pg<uint8_t>, grid, block, 0, c->stream[me], d, dst_off, src_off, nelems, me, pe, g); break;
    case 2: hipLaunchKernelGGL(shmk_scalar_pg<uint16_t>, grid, block, 0, c->stream[me], d, dst_off, src_off, nelems, me, pe, g); break;
    case 4: hipLaunchKernelGGL(shmk_scalar_pg<uint32_t>, grid, block, 0, c->stream[me], d, dst_off, src_off, nelems, me, pe, g); break;
    default: hipLaunchKernelGGL(shmk_scalar_pg<uint64_t>, grid, block, 0, c->stream[me], d, dst_off, src_off, nelems, me, pe, g); break;
    }
    return launched("scalar put/get");
}

int shm_launch_wave_exchange(shm_ctx *c, int me, int pe, uint64_t dst_off, uint64_t src_off, uint64_t back_off, size_t n, int n_waves,
                             uint64_t flag_off, uint64_t out_off)
{
    if (int r = check_ctx(c)) return r;
    if (int r = rma_args(c, me, pe, dst_off, src_off, n)) return r;
    if (n_waves < 1 || n_waves > 4096) return fail(SHM_EINVAL, "n_waves outside 1..4096");
    if (int r = check_range(c, back_off, n, "back buffer")) return r;
    if (int r = check_range(c, flag_off, 8ull * n_waves, "flags")) return r;
    if (int r = check_range(c, out_off, 8ull * n_waves, "fetched values")) return r;
    if ((flag_off | out_off) & 7) return fail(SHM_EINVAL, "flag and out offsets must be 8-byte aligned");
    // on PE pe: destination, back buffer, flags and out words are pairwise disjoint (and the source too if me == pe)
    struct span {
        uint64_t off;
        size_t len;
    };
    const span on_pe[5] = {{dst_off, n}, {back_off, n}, {flag_off, 8ull * n_waves}, {out_off, 8ull * n_waves}, {src_off, me == pe ? n : 0}};
    for (int i = 0; i < 5; ++i)
        for (int j = i + 1; j < 5; ++j)
            if (on_pe[i].len && on_pe[j].len && on_pe[i].off < on_pe[j].off + on_pe[j].len && on_pe[j].off < on_pe[i].off + on_pe[i].len)
                return fail(SHM_EINVAL, "buffers overlap on PE %d", pe);
    if (c->no_device) return no_device("shm_launch_wave_exchange");
    if (int r = begin_pe_launch(c, me)) return r;
    int per_cu = 0;
    HIP_TRY(hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, shmk_wave_exchange, SHMK_WG, 0));
    const long long groups = 2ll * ((n_waves + 3) / 4);
    if (groups > static_cast<long long>(per_cu) * c->num_cu)
        return fail(SHM_EINVAL, "%lld groups cannot all be resident (%d CUs x %d)", groups, c->num_cu, per_cu);
    hipLaunchKernelGGL(shmk_wave_exchange, dim3(static_cast<unsigned>(groups)), dim3(SHMK_WG), 0, c->stream[me], dev_view(c), dst_off,
                       src_off, back_off, n, n_waves, flag_off, out_off, me, pe);
    return launched("wave exchange");
}

int shm_launch_thread_rma(shm_ctx *c, int me, int pe, uint64_t dst_off, uint64_t src_off, size_t n, int is_get, int reps,
                          uint64_t *dev_ticks)
{
    if (int r = check_ctx(c)) return r;
    if (int r = rma_args(c, me, pe, dst_off, src_off, n)) return r;
    if (reps < 1 || reps > (1 << 20)) return fail(SHM_EINVAL, "reps outside 1..2^20");
    if (c->no_device) return no_device("shm_launch_thread_rma");
    if (int r = begin_pe_launch(c, me)) return r;
    hipLaunchKernelGGL(shmk_thread_rma, dim3(1), dim3(64), 0, c->stream[me], dev_view(c), dst_off, src_off, n, me, pe, is_get ? 1 : 0,
                       reps, reinterpret_cast<unsigned long long *>(dev_ticks));
    return launched("single-thread transfer");
}

namespace {
int launch_strided(shm_ctx *c, int me, int pe, uint64_t dst_off, uint64_t src_off, int64_t dst_stride, int64_t src_stride, size_t nelems,
                   int elem_bytes, int n_wg, int is_get)
{
    if (int r = check_ctx(c)) return r;
    if (int r = check_pe(c, me, "calling PE")) return r;
    if (int r = check_pe(c, pe, "target PE")) return r;
    if (elem_bytes != 1 && elem_bytes != 2 && elem_bytes != 4 && elem_bytes != 8 && elem_bytes != 16)
        return fail(SHM_EINVAL, "element size %d is not 1, 2, 4, 8 or 16", elem_bytes);
    if (dst_stride < 1 || src_stride < 1) return fail(SHM_EINVAL, "strides are counted in elements and are at least 1");
    if ((dst_off | src_off) % static_cast<uint64_t>(elem_bytes)) return fail(SHM_EINVAL, "strided transfers need element-aligned offsets");
    if (n_wg < 0 || n_wg > 65535) return fail(SHM_EINVAL, "n_wg outside 0..65535");
    const uint64_t e = static_cast<uint64_t>(elem_bytes), limit = c->user_bytes / e + 1;
    uint64_t dspan = 0, sspan = 0;
    if (nelems) {
        // (nelems - 1) * stride + 1 elements, computed without overflow; one element has no stride to speak of
        if (nelems - 1 > limit || (nelems - 1) * static_cast<unsigned __int128>(dst_stride) > limit ||
            (nelems - 1) * static_cast<unsigned __int128>(src_stride) > limit)
            return fail(SHM_ERANGE, "the strided transfer leaves the heap");
        dspan = ((nelems - 1) * static_cast<uint64_t>(dst_stride) + 1) * e;
        sspan = ((nelems - 1) * static_cast<uint64_t>(src_stride) + 1) * e;
    }
    if (int r = check_range(c, dst_off, dspan, "destination")) return r;
    if (int r = check_range(c, src_off, sspan, "source")) return r;
    if (me == pe && nelems && src_off < dst_off + dspan && dst_off < src_off + sspan)
        return fail(SHM_EINVAL, "source and destination overlap on PE %d", me);
    if (c->no_device) return no_device("strided transfer");
    if (int r = begin_pe_launch(c, me)) return r;
    if (nelems == 0) return SHM_OK;
    hipLaunchKernelGGL(shmk_strided, dim3(n_wg ? n_wg : 1), dim3(n_wg ? SHMK_WG : 64), 0, c->stream[me], dev_view(c), dst_off, src_off,
                       static_cast<size_t>(dst_stride), static_cast<size_t>(src_stride), nelems, static_cast<uint32_t>(elem_bytes), me, pe,
                       is_get, n_wg ? 0 : 1);
    return launched("strided transfer");
}
}  // namespace

int shm_launch_iput(shm_ctx *c, int me, int pe, uint64_t dst_off, uint64_t src_off, int64_t dst_stride, int64_t src_stride, size_t nelems,
                    int elem_bytes, int n_wg)
{
    return launch_strided(c, me, pe, dst_off, src_off, dst_stride, src_stride, nelems, elem_bytes, n_wg, 0);
}

int shm_launch_iget(shm_ctx *c, int me, int pe, uint64_t dst_off, uint64_t src_off, int64_t dst_stride, int64_t src_stride, size_t nelems,
                    int elem_bytes, int n_wg)
{
    return launch_strided(c, me, pe, dst_off, src_off, dst_stride, src_stride, nelems, elem_bytes, n_wg, 1);
}

int shm_launch_offload_nop(shm_ctx *c, int me, int n_wg, int reps, int blocking, uint64_t *dev_ticks)
{
    if (int r = check_ctx(c)) return r;
    if (int r = check_pe(c, me, "calling PE")) return r;
    if (n_wg < 1 || n_wg > 4096) return fail(SHM_EINVAL, "n_wg outside 1..4096");
    if (reps < 1 || reps > (1 << 20)) return fail(SHM_EINVAL, "reps outside 1..2^20");
    if (!dev_ticks) return fail(SHM_EINVAL, "null tick buffer");
    if (c->no_device) return no_device("shm_launch_offload_nop");
    if (!c->proxy.running()) return fail(SHM_EINVAL, "the host proxy is not running (shm_proxy_start)");
    if (int r = begin_pe_launch(c, me)) return r;
    hipLaunchKernelGGL(shmk_offload_nop, dim3(n_wg), dim3(SHMK_WG), 0, c->stream[me], dev_view(c), me, reps, blocking,
                       reinterpret_cast<unsigned long long *>(dev_ticks));
    return launched("offload ring test");
}

int shm_wall_clock_khz(const shm_ctx *c)
{
    if (int r = check_ctx(c)) return r;
    return static_cast<int>(c->ticks_per_us * 1000);
}

int shm_launch_wg_put_signal(shm_ctx *c, int me, int pe, uint64_t dst_off, uint64_t src_off, size_t n, uint64_t sig_off,
                             uint64_t sig_val, int sig_op, int n_wg)
{
    if (int r = check_ctx(c)) return r;
    if (int r = rma_args(c, me, pe, dst_off, src_off, n)) return r;
    if (int r = check_word(c, sig_off, "signal")) return r;
    if (sig_op != SHM_SIGNAL_SET && sig_op != SHM_SIGNAL_ADD) return fail(SHM_EINVAL, "signal op %d is neither SET nor ADD", sig_op);
    if (int r = check_n_wg(n_wg)) return r;
    if (n && sig_off + 8 > dst_off && sig_off < dst_off + n)
        return fail(SHM_EINVAL, "signal word lies inside the destination");
    if (c->no_device) return no_device("shm_launch_wg_put_signal");
    if (int r = begin_pe_launch(c, me)) return r;
    uint64_t *arrive = nullptr;
    if (n_wg > 1) arrive = reinterpret_cast<uint64_t *>(shm_ptr(c, c->user_bytes, me)) + take_slots(c, me, 1);
    hipLaunchKernelGGL(shmk_wg_put_signal, dim3(n_wg), dim3(SHMK_WG), 0, c->stream[me], dev_view(c), me, pe, dst_off, src_off, n,
                       sig_off, sig_val, sig_op, arrive);
    return launched("put with signal");
}

int shm_launch_signal_wait_until(shm_ctx *c, int me, uint64_t sig_off, int cmp, uint64_t val, uint64_t *dev_out)
{
    if (int r = check_ctx(c)) return r;
    if (int r = check_pe(c, me, "calling PE")) return r;
    if (int r = check_word(c, sig_off, "signal")) return r;
    if (cmp < SHM_CMP_EQ || cmp > SHM_CMP_LE) return fail(SHM_EINVAL, "unknown comparison %d", cmp);
    if (c->no_device) return no_device("shm_launch_signal_wait_until");
    if (int r = begin_pe_launch(c, me)) return r;
    hipLaunchKernelGGL(shmk_signal_wait, dim3(1), dim3(SHMK_WG), 0, c->stream[me], dev_view(c), me, sig_off, cmp, val, dev_out);
    return launched("signal wait");
}

int shm_launch_sync_set(shm_ctx *c, int me, uint64_t ivars_off, size_t nelems, const int *dev_status, int kind, int cmp, int64_t val,
                        uint64_t *dev_out)
{
    if (int r = check_ctx(c)) return r;
    if (int r = check_pe(c, me, "calling PE")) return r;
    if (kind < SHM_SYNC_WAIT || kind > SHM_SYNC_TEST_SOME) return fail(SHM_EINVAL, "unknown synchronisation kind %d", kind);
    if (cmp < SHM_CMP_EQ || cmp > SHM_CMP_LE) return fail(SHM_EINVAL, "unknown comparison %d", cmp);
    const bool single = kind == SHM_SYNC_WAIT || kind == SHM_SYNC_TEST;
    if (single && nelems == 0) nelems = 1;
    if (nelems > c->user_bytes / 8) return fail(SHM_ERANGE, "the variables leave the heap");
    if (int r = check_range(c, ivars_off, 8 * nelems, "variables")) return r;
    if (ivars_off & 7) return fail(SHM_EINVAL, "variables must be 8-byte aligned");
    if (!dev_out) return fail(SHM_EINVAL, "null result buffer");
    if (c->no_device) return no_device("shm_launch_sync_set");
    if (int r = begin_pe_launch(c, me)) return r;
    hipLaunchKernelGGL(shmk_sync_set, dim3(1), dim3(64), 0, c->stream[me], dev_view(c), me, ivars_off, nelems, dev_status, kind, cmp,
                       static_cast<long long>(val), reinterpret_cast<unsigned long long *>(dev_out));
    return launched("point-to-point synchronisation");
}

int shm_launch_amo(shm_ctx *c, int me, int pe, uint64_t off, int op, int64_t operand, int64_t cond, int64_t *dev_out)
{
    if (int r = check_ctx(c)) return r;
    if (int r = check_pe(c, me, "calling PE")) return r;
    if (int r = check_pe(c, pe, "target PE")) return r;
    if (int r = check_word(c, off, "atomic target")) return r;
    if (op < SHM_AMO_FETCH || op > SHM_AMO_INC) return fail(SHM_EINVAL, "unknown atomic op %d", op);
    if (c->no_device) return no_device("shm_launch_amo");
    if (int r = begin_pe_launch(c, me)) return r;
    hipLaunchKernelGGL(shmk_amo, dim3(1), dim3(64), 0, c->stream[me], dev_view(c), pe, off, op, operand, cond, dev_out);
    return launched("atomic");
}

int shm_launch_pingflag(shm_ctx *c, uint64_t data_off, uint64_t back_off, size_t n, uint64_t flag_off)
{
    if (int r = check_ctx(c)) return r;
    if (c->npes < 2) return fail(SHM_EPE, "needs at least 2 PEs");
    if (int r = check_range(c, data_off, n, "data")) return r;
    if (int r = check_range(c, back_off, n, "get-back buffer")) return r;
    if (int r = check_word(c, flag_off, "flag")) return r;
    if (overlaps(data_off, back_off, n)) return fail(SHM_EINVAL, "data and get-back buffer overlap");
    if ((flag_off + 8 > data_off && flag_off < data_off + n) || (flag_off + 8 > back_off && flag_off < back_off + n))
        return fail(SHM_EINVAL, "flag lies inside a data buffer");
    if (c->no_device) return no_device("shm_launch_pingflag");
    if (int r = drain_all_engines(c)) return r;
    if (int r = begin_pe_launch(c, 0)) return r;
    if (int r = begin_pe_launch(c, 1)) return r;
    const shm_dev_ctx d = dev_view(c);
    // The producer is enqueued first: it never waits, so the consumer's bounded wait always ends.
    hipLaunchKernelGGL(shmk_ping_producer, dim3(1), dim3(SHMK_WG), 0, c->stream[0], d, data_off, n, flag_off);
    if (int r = launched("ping producer")) return r;
    hipLaunchKernelGGL(shmk_ping_consumer, dim3(1), dim3(SHMK_WG), 0, c->stream[1], d, data_off, back_off, n, flag_off);
    return launched("ping consumer");
}

namespace {

// Address of this device's copy of `scratch` (asked for once per device, with that device current).
int static_scratch(unsigned long long **out)
{
    int dev = 0;
    HIP_TRY(hipGetDevice(&dev));
    if (dev < 0 || dev >= MAX_DEVICES) return fail(SHM_EHIP, "device %d is beyond the %d devices the library keeps scratch addresses for", dev, MAX_DEVICES);
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void *p = nullptr;
        HIP_TRY(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
        if (!p) return fail(SHM_EHIP, "hipGetSymbolAddress returned no address for the scratch array");
        g_scratch_ptr[dev] = static_cast<unsigned long long *>(p);
    }
    *out = g_scratch_ptr[dev];
    return SHM_OK;
}

// static_counters: the arrival counters come from the library's static scratch array (and are cleared
// by a kernel first) instead of from the heap's tail.
int ring_pipeline(shm_ctx *c, uint64_t src_off, uint64_t slot_off, uint64_t sig_off, uint64_t acc_off, size_t chunk_bytes, int n_chunks,
                  int n_wg_prod, int n_wg_cons, int n_sig, bool static_counters)
{
    if (int r = check_ctx(c)) return r;
    if (static_counters && n_chunks > SHM_STATIC_RING_MAX_CHUNKS)
        return fail(SHM_EINVAL, "n_chunks %d exceeds the %d chunks the static scratch array has arrival counters for", n_chunks,
                    SHM_STATIC_RING_MAX_CHUNKS);
    if (chunk_bytes == 0 || chunk_bytes % 16) return fail(SHM_EINVAL, "chunk_bytes must be a positive multiple of 16");
    if (n_chunks < 1 || static_cast<uint32_t>(n_chunks) > ARRIVE_SLOTS) return fail(SHM_EINVAL, "n_chunks outside 1..%u", ARRIVE_SLOTS);
    if (n_wg_prod < 1 || n_wg_cons < 1 || n_wg_prod > MAX_N_WG || n_wg_cons > MAX_N_WG)
        return fail(SHM_EINVAL, "producer and consumer groups per PE outside 1..%d", MAX_N_WG);
    if (chunk_bytes > c->user_bytes / n_chunks) return fail(SHM_ERANGE, "chunks leave the heap");
    const size_t total = chunk_bytes * n_chunks;
    if (int r = check_range(c, src_off, total, "chunk source")) return r;
    if (int r = check_range(c, slot_off, total, "landing slots")) return r;
    if (int r = check_range(c, acc_off, chunk_bytes * 2, "accumulator")) return r;
    if (n_sig != 1 && !(n_sig == n_wg_prod && n_sig == n_wg_cons))
        return fail(SHM_EINVAL, "n_sig must be 1 or equal to both n_wg_prod and n_wg_cons");
    if (int r = check_range(c, sig_off, 8ull * n_sig, "signals")) return r;
    if (sig_off & 7) return fail(SHM_EINVAL, "signal words must be 8-byte aligned");
    if ((src_off | slot_off | acc_off) & 15) return fail(SHM_EINVAL, "offsets must be 16-byte aligned");
    if (overlaps(src_off, slot_off, total) || (acc_off < slot_off + total && slot_off < acc_off + 2 * chunk_bytes) ||
        (acc_off < src_off + total && src_off < acc_off + 2 * chunk_bytes))
        return fail(SHM_EINVAL, "source, slots and accumulator must be disjoint");
    {
        const uint64_t sig_end = sig_off + 8ull * n_sig;
        if ((sig_off < src_off + total && src_off < sig_end) || (sig_off < slot_off + total && slot_off < sig_end) ||
            (sig_off < acc_off + 2 * chunk_bytes && acc_off < sig_end))
            return fail(SHM_EINVAL, "signal words lie inside a data buffer");
    }
    const size_t nvec = chunk_bytes / 16;
    if ((nvec + n_wg_cons - 1) / n_wg_cons > static_cast<size_t>(SHMK_WG) * SHMK_RING_VPT)
        return fail(SHM_EINVAL, "n_wg_cons too small: a consumer group holds at most %d bytes of a chunk", SHMK_WG * SHMK_RING_VPT * 16);
    if (c->no_device) return no_device("shm_launch_ring_pipeline");
    if (int r = drain_all_engines(c)) return r;
    int per_cu = 0;
    const bool lanes = n_sig > 1 || (n_wg_prod == 1 && n_wg_cons == 1);
    // producer shares of 32-128 KiB per chunk take the form that keeps two 64 KiB blocks in registers
    const size_t pper = (nvec + n_wg_prod - 1) / n_wg_prod;
    const bool deep = !lanes && pper > static_cast<size_t>(SHMK_WG) * SHMK_RING_VPT && pper <= 2u * SHMK_WG * SHMK_RING_DEEP_VPT;
    auto kernel = lanes ? shmk_ring<1, 0> : deep ? shmk_ring<0, 1> : shmk_ring<0, 0>;
    HIP_TRY(hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, kernel, SHMK_WG, 0));
    const long long groups = static_cast<long long>(c->npes) * (n_wg_prod + n_wg_cons);
    if (deep && groups > static_cast<long long>(per_cu) * c->num_cu) {       // too many groups for its registers: the plain form
        kernel = shmk_ring<0, 0>;
        HIP_TRY(hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, kernel, SHMK_WG, 0));
    }
    if (groups > static_cast<long long>(per_cu) * c->num_cu)
        return fail(SHM_EINVAL, "%lld groups cannot all be resident (%d CUs x %d); consumers would wait on groups that never start",
                    groups, c->num_cu, per_cu);
    // one arrival counter per chunk, same slot range on every PE
    uint64_t *arrive_pe0 = nullptr;
    uint64_t arrive_stride = 0;
    unsigned long long *static_ptr = nullptr;
    if (static_counters) {
        if (int r = static_scratch(&static_ptr)) return r;
        arrive_pe0 = reinterpret_cast<uint64_t *>(static_ptr);
        arrive_stride = SHM_STATIC_RING_MAX_CHUNKS;
    } else {
        uint32_t first = 0;
        for (int p = 0; p < c->npes; ++p) c->next_slot[p] = 0;
        for (int p = 0; p < c->npes; ++p) first = take_slots(c, p, n_chunks);
        arrive_pe0 = reinterpret_cast<uint64_t *>(c->base + c->user_bytes) + first;
        arrive_stride = c->part_bytes / 8;
    }
    if (c->team_sync)
        if (int r = team_join(c)) return r;
    if (static_counters) {
        // the array keeps what the last call left (a call that ran into a wait bound may have left counts): start from zero
        const size_t words = static_cast<size_t>(c->npes) * SHM_STATIC_RING_MAX_CHUNKS;
        hipLaunchKernelGGL(shmk_clear_words, dim3(static_cast<unsigned>((words + SHMK_WG - 1) / SHMK_WG)), dim3(SHMK_WG), 0, c->stream[0],
                           static_ptr, words);
        if (int r = launched("clearing the static arrival counters")) return r;
    }
    hipLaunchKernelGGL(kernel, dim3(static_cast<unsigned>(groups)), dim3(SHMK_WG), 0, c->stream[0], dev_view(c), src_off, slot_off, sig_off,
                       acc_off, chunk_bytes, n_chunks, n_wg_prod, n_wg_cons, arrive_pe0, arrive_stride);
    if (int r = launched("ring pipeline")) return r;
    if (c->team_sync)
        if (int r = team_fork(c)) return r;
    return SHM_OK;
}

}  // namespace

int shm_launch_ring_pipeline(shm_ctx *c, uint64_t src_off, uint64_t slot_off, uint64_t sig_off, uint64_t acc_off, size_t chunk_bytes,
                             int n_chunks, int n_wg_prod, int n_wg_cons, int n_sig)
{
    return ring_pipeline(c, src_off, slot_off, sig_off, acc_off, chunk_bytes, n_chunks, n_wg_prod, n_wg_cons, n_sig, false);
}

int shm_launch_ring_pipeline_static(shm_ctx *c, uint64_t src_off, uint64_t slot_off, uint64_t sig_off, uint64_t acc_off, size_t chunk_bytes,
                                    int n_chunks, int n_wg_prod, int n_wg_cons, int n_sig)
{
    return ring_pipeline(c, src_off, slot_off, sig_off, acc_off, chunk_bytes, n_chunks, n_wg_prod, n_wg_cons, n_sig, true);
}

int shm_launch_amo_storm(shm_ctx *c, uint64_t ctr_off, int n_ctr, const uint16_t *dev_targets, uint64_t n_items, int ops_per_item,
                         int kind, int64_t *dev_fetched, uint64_t *dev_checksum)
{
    if (int r = check_ctx(c)) return r;
    if (n_ctr < 1 || static_cast<long long>(n_ctr) * c->npes > 65536) return fail(SHM_EINVAL, "npes * n_ctr must be 1..65536 (16-bit targets)");
    if (int r = check_range(c, ctr_off, 8ull * n_ctr, "counters")) return r;
    if (ctr_off & 7) return fail(SHM_EINVAL, "counters must be 8-byte aligned");
    if (!dev_targets) return fail(SHM_EINVAL, "null target table");
    if (reinterpret_cast<uintptr_t>(dev_targets) & 15) return fail(SHM_EINVAL, "target table must be 16-byte aligned");
    if (ops_per_item < 1 || ops_per_item > 4096) return fail(SHM_EINVAL, "ops_per_item outside 1..4096");
    if (kind < SHM_STORM_FETCH_ADD || kind > SHM_STORM_FETCH_ADD_WG) return fail(SHM_EINVAL, "unknown storm kind %d", kind);
    const bool batched = kind == SHM_STORM_FETCH_ADD_WG;
    const size_t table_bytes = 8ull * n_ctr * c->npes;            // the batched kind's table in LDS
    if (batched && table_bytes > SHMK_STORM_TABLE_BYTES)
        return fail(SHM_EINVAL, "the batched storm keeps npes * n_ctr <= %d counters in LDS", static_cast<int>(SHMK_STORM_TABLE_BYTES / 8));
    const uint64_t groups = (n_items + SHMK_WG - 1) / SHMK_WG;
    if (n_items == 0 || groups >= (1ull << 24)) return fail(SHM_EINVAL, "n_items outside 1..2^32-256 (one grid holds fewer than 2^32 threads)");
    if (c->no_device) return no_device("shm_launch_amo_storm");
    if (int r = drain_all_engines(c)) return r;
    if (c->team_sync)
        if (int r = team_join(c)) return r;
    const shm_dev_ctx d = dev_view(c);
    const dim3 grid(static_cast<unsigned>(groups)), block(SHMK_WG);
    hipStream_t s = c->stream[0];
    switch (kind) {
    case SHM_STORM_FETCH_ADD_WG: {
        // more LDS than a kernel gets without asking; so one group per compute unit, and no more groups than those
        HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void *>(shmk_amo_storm_wg), hipFuncAttributeMaxDynamicSharedMemorySize,
                                    static_cast<int>(SHMK_STORM_TABLE_BYTES)));
        const uint64_t rounds = (n_items + SHMK_STORM_WG - 1) / SHMK_STORM_WG;
        const uint64_t want_groups = std::min<uint64_t>(rounds, std::max(1, c->num_cu));
        const uint64_t items_per_group = (rounds + want_groups - 1) / want_groups * SHMK_STORM_WG;
        const dim3 big_grid(static_cast<unsigned>((n_items + items_per_group - 1) / items_per_group)), big_block(SHMK_STORM_WG);
        hipLaunchKernelGGL(shmk_amo_storm_wg, big_grid, big_block, table_bytes, s, d, ctr_off, n_ctr, dev_targets, n_items, ops_per_item,
                           dev_fetched, dev_checksum, items_per_group);
        break;
    }
    case SHM_STORM_FETCH_ADD:
        hipLaunchKernelGGL(shmk_amo_storm<0>, grid, block, 0, s, d, ctr_off, n_ctr, dev_targets, n_items, ops_per_item, dev_fetched, dev_checksum);
        break;
    case SHM_STORM_ADD:
        hipLaunchKernelGGL(shmk_amo_storm<1>, grid, block, 0, s, d, ctr_off, n_ctr, dev_targets, n_items, ops_per_item, dev_fetched, dev_checksum);
        break;
    case SHM_STORM_CSWAP_LOOP:
        hipLaunchKernelGGL(shmk_amo_storm<2>, grid, block, 0, s, d, ctr_off, n_ctr, dev_targets, n_items, ops_per_item, dev_fetched, dev_checksum);
        break;
    default:
        hipLaunchKernelGGL(shmk_amo_storm<3>, grid, block, 0, s, d, ctr_off, n_ctr, dev_targets, n_items, ops_per_item, dev_fetched, dev_checksum);
        break;
    }
    if (int r = launched("atomic storm")) return r;
    if (c->team_sync)
        if (int r = team_fork(c)) return r;
    return SHM_OK;
}

int shm_launch_fcollect(shm_ctx *c, uint64_t dst_off, uint64_t src_off, size_t bytes_per_pe, int n_wg, int path)
{
    if (int r = check_ctx(c)) return r;
    if (bytes_per_pe > c->user_bytes / c->npes) return fail(SHM_ERANGE, "destination of %d blocks leaves the heap", c->npes);
    const size_t total = bytes_per_pe * c->npes;
    if (int r = check_range(c, src_off, bytes_per_pe, "source")) return r;
    if (int r = check_range(c, dst_off, total, "destination")) return r;
    if (bytes_per_pe && src_off < dst_off + total && dst_off < src_off + bytes_per_pe)
        return fail(SHM_EINVAL, "source and destination overlap");
    if (int r = check_team_grid(c, n_wg)) return r;
    int use;
    if (int r = resolve_collective_path(c, SHM_COLL_FCOLLECT, path, bytes_per_pe, n_wg, &use)) return r;
    if (c->no_device) return no_device("shm_launch_fcollect");
    if (bytes_per_pe == 0) return team_order_only(c);
    if (int r = drain_all_engines(c)) return r;
    if (use != SHM_PATH_LDST) {
        if (c->team_sync) {
            if (int r = team_join(c)) return r;
            if (int r = team_fork(c)) return r;
        }
        for (int j = 0; j < c->npes; ++j)          // destination index varies fastest across streams
            for (int p = 0; p < c->npes; ++p) {
                const int q = (p + 1 + j) % c->npes;
                if (int r = transfer_copy(c, use, p, q, dst_off + static_cast<uint64_t>(p) * bytes_per_pe, p, src_off, bytes_per_pe))
                    return r;
            }
        if (c->team_sync) {
            // the engines are not on the streams: only the host can put later work of OTHER PEs behind them
            if (use == SHM_PATH_SDMA)
                if (int r = drain_all_engines(c)) return r;
            if (int r = team_join(c)) return r;
            if (int r = team_fork(c)) return r;
        }
        return SHM_OK;
    }
    if (c->team_sync)
        if (int r = team_join(c)) return r;
    // A long block is pushed fastest by about one group per compute unit, each streaming many tiles
    // (measured, 8 PEs x 64 MiB: 32 groups per PE 0.80 ms, 256 groups 0.85 ms, 1024 groups 0.87 ms).
    // Which group moves which tile cannot be observed, so from 16 tiles per group on the launcher
    // runs that many groups, never more than it was asked for.
    const int per_cu = c->num_cu / c->npes > 0 ? c->num_cu / c->npes : 1;
    if (n_wg > per_cu && bytes_per_pe / TILE_BYTES >= 16u * static_cast<size_t>(per_cu)) n_wg = per_cu;
    // From 8 MiB per PE and 6 PEs on (fcollect_by_ticket), those groups draw quarter-tile pieces (16 KiB) of their PE's block
    // by ticket, in address order, and store every column to the destinations in turn (measured, % of
    // the HBM roofline, fixed tiles -> tickets: 8 PEs x 8 / 16 / 64 MiB 62.9 -> 73.6, 65.5 -> 77.8, 76.9 -> 80.7
    // -- the write-only ceiling of this chip is 81 % --; 16 PEs 63.1 -> 73.5, 69.8 -> 74.5, 71.2 -> 74.0; with
    // other numbers of groups -- 8 PEs: 24 groups 69 %, 40 and more 76-77 % -- nothing is gained; fewer PEs: fcollect_by_ticket).
    uint64_t pair = 0;
    if (((dst_off | src_off | bytes_per_pe) & 15) == 0 && fcollect_by_ticket(c, bytes_per_pe) && n_wg >= per_cu) {
        n_wg = per_cu;
        pair = ticket_pair_off(c, SHMD_TICKET_COLL);
    }
    // on tiles, from 8 MiB per PE, a whole number of groups per compute unit in all (6 PEs x 24 MiB asked of 48 / 70
    // groups: 59.8 / 65.3 -> 73.1 / 73.6 % of the HBM roofline; at 6 MiB mixed)
    if (!pair && bytes_per_pe >= FCOLLECT_TICKETS_MIN_BYTES) n_wg = static_cast<int>(balanced_groups(c, static_cast<unsigned>(n_wg), c->npes));
    const dim3 grid(n_wg, c->npes), block(SHMK_WG);
    if (((dst_off | src_off | bytes_per_pe) & 15) == 0) {
        if (c->npes == 8)
            hipLaunchKernelGGL((shmk_fcollect_vec<2, 8>), grid, block, 0, c->stream[0], dev_view(c), dst_off, src_off, bytes_per_pe, pair);
        else
            hipLaunchKernelGGL((shmk_fcollect_vec<2, 0>), grid, block, 0, c->stream[0], dev_view(c), dst_off, src_off, bytes_per_pe, pair);
    } else
        hipLaunchKernelGGL(shmk_fcollect_any, grid, block, 0, c->stream[0], dev_view(c), dst_off, src_off, bytes_per_pe);
    if (int r = launched("fcollect")) return r;
    if (c->team_sync)
        if (int r = team_fork(c)) return r;
    return SHM_OK;
}

int shm_launch_collect(shm_ctx *c, uint64_t dst_off, uint64_t src_off, const size_t *nbytes_per_pe, int n_wg)
{
    if (int r = check_ctx(c)) return r;
    if (!nbytes_per_pe) return fail(SHM_EINVAL, "null size array");
    shmk_collect_table t;
    memset(&t, 0, sizeof t);
    size_t total = 0, largest = 0;
    for (int p = 0; p < c->npes; ++p) {
        if (nbytes_per_pe[p] > c->user_bytes - total) return fail(SHM_ERANGE, "the concatenation leaves the heap");
        t.at[p] = total;
        t.nbytes[p] = nbytes_per_pe[p];
        total += nbytes_per_pe[p];
        if (nbytes_per_pe[p] > largest) largest = nbytes_per_pe[p];
    }
    if (int r = check_range(c, dst_off, total, "destination")) return r;
    if (int r = check_range(c, src_off, largest, "source")) return r;
    if (total && largest && src_off < dst_off + total && dst_off < src_off + largest)
        return fail(SHM_EINVAL, "source and destination overlap");
    if (int r = check_team_grid(c, n_wg)) return r;
    if (c->no_device) return no_device("shm_launch_collect");
    if (int r = drain_all_engines(c)) return r;
    if (total == 0) return team_order_only(c);
    if (c->team_sync)
        if (int r = team_join(c)) return r;
    // Blocks that all lie and end on multiples of 16 bytes are pushed like fcollect's: about a group per
    // compute unit for long blocks, and from 8 MiB (the largest block) and 8 PEs on pieces by ticket
    // (measured, 8 PEs, % of the HBM roofline, 32 / 256 / 1024 groups per PE asked -> now: blocks of 64 MiB
    // 60.5 / 61.0 / 47.2 -> 80.6, of 48 MiB and up to 109 KiB more 59.0 / 61.5 / 50.4 -> 71.2, of 8 MiB and up to
    // 28 KiB more 62.9 / 64.5 / 68.8 -> 72.9).  Otherwise the kernel pushes the blocks that do the same way
    // and the others the general way (the source read once as aligned words, every vector put together and
    // stored to all PEs), with the groups it was asked for (blocks of 40-61 MiB that begin at odd bytes:
    // 42 / 61 / 61 %; 19 / 35 / 39 % as a put per destination).
    bool aligned = ((dst_off | src_off) & 15) == 0;
    for (int p = 0; p < c->npes; ++p) aligned = aligned && ((t.at[p] | t.nbytes[p]) & 15) == 0;
    const int per_cu = c->num_cu / c->npes > 0 ? c->num_cu / c->npes : 1;
    if (aligned && n_wg > per_cu && largest / TILE_BYTES >= 16u * static_cast<size_t>(per_cu)) n_wg = per_cu;
    uint64_t pair = 0;
    if (aligned && fcollect_by_ticket(c, largest) && n_wg >= per_cu) {
        n_wg = per_cu;
        pair = ticket_pair_off(c, SHMD_TICKET_COLL);
    }
    if (aligned && !pair && largest >= FCOLLECT_TICKETS_MIN_BYTES)      // as fcollect on tiles: a whole number of groups per compute unit
        n_wg = static_cast<int>(balanced_groups(c, static_cast<unsigned>(n_wg), c->npes));
    if (c->npes == 8)
        hipLaunchKernelGGL(shmk_collect<8>, dim3(n_wg, c->npes), dim3(SHMK_WG), 0, c->stream[0], dev_view(c), dst_off, src_off, t, pair);
    else
        hipLaunchKernelGGL(shmk_collect<0>, dim3(n_wg, c->npes), dim3(SHMK_WG), 0, c->stream[0], dev_view(c), dst_off, src_off, t, pair);
    if (int r = launched("collect")) return r;
    if (c->team_sync)
        if (int r = team_fork(c)) return r;
    return SHM_OK;
}

int shm_launch_reduce(shm_ctx *c, uint64_t dst_off, uint64_t src_off, size_t nelems, int dtype, int op, int n_wg, int algo)
{
    if (int r = check_ctx(c)) return r;
    size_t elem = 0;
    const reduce_kernel k = pick_reduce(dtype, op, algo == SHM_REDUCE_SPLIT, &elem);
    if (elem == 0) return fail(SHM_EINVAL, "unknown element type %d", dtype);
    if (op < SHM_OP_MIN || op > SHM_OP_XOR) return fail(SHM_EINVAL, "unknown reduction %d", op);
    if (!k) return fail(SHM_EINVAL, "and/or/xor are defined for integer types only");
    if (algo != SHM_REDUCE_DUPLICATE && algo != SHM_REDUCE_SPLIT) return fail(SHM_EINVAL, "unknown reduction algorithm %d", algo);
    if (nelems > c->user_bytes / elem) return fail(SHM_ERANGE, "vector leaves the heap");
    if (int r = check_range(c, src_off, nelems * elem, "source")) return r;
    if (int r = check_range(c, dst_off, nelems * elem, "destination")) return r;
    if ((src_off | dst_off) & 15) return fail(SHM_EINVAL, "reduction buffers must be 16-byte aligned");
    if (overlaps(dst_off, src_off, nelems * elem)) return fail(SHM_EINVAL, "source and destination overlap");
    if (int r = check_team_grid(c, n_wg)) return r;
    if (c->no_device) return no_device("shm_launch_reduce");
    if (int r = drain_all_engines(c)) return r;
    if (nelems == 0) return team_order_only(c);
    if (c->team_sync)
        if (int r = team_join(c)) return r;
    uint64_t pair = 0;
    if (algo == SHM_REDUCE_SPLIT) n_wg = split_reduce_groups(c, nelems / (16 / elem), n_wg, &pair);
    else n_wg = duplicate_reduce_groups(c, nelems * elem, n_wg);
    hipLaunchKernelGGL(k, dim3(n_wg, c->npes), dim3(SHMK_WG), 0, c->stream[0], dev_view(c), dst_off, src_off, nelems, pair);
    if (int r = launched("reduce")) return r;
    if (c->team_sync)
        if (int r = team_fork(c)) return r;
    return SHM_OK;
}

int shm_launch_barrier_exchange(shm_ctx *c, uint64_t dst_off, uint64_t src_off, uint64_t acc_off, size_t n, int rounds)
{
    if (int r = check_ctx(c)) return r;
    if (rounds < 1 || rounds > c->npes) return fail(SHM_EINVAL, "rounds outside 1..npes");
    if (n > c->user_bytes / c->npes) return fail(SHM_ERANGE, "slots leave the heap");
    if (int r = check_range(c, src_off, n, "source")) return r;
    if (int r = check_range(c, dst_off, n * c->npes, "slots")) return r;
    if (int r = check_range(c, acc_off, n * rounds, "result")) return r;
    const size_t dn = n * c->npes, an = n * rounds;
    if (n && ((src_off < dst_off + dn && dst_off < src_off + n) || (src_off < acc_off + an && acc_off < src_off + n) ||
              (dst_off < acc_off + an && acc_off < dst_off + dn)))
        return fail(SHM_EINVAL, "source, slots and result must be disjoint");
    if (c->no_device) return no_device("shm_launch_barrier_exchange");
    if (int r = drain_all_engines(c)) return r;
    if (c->team_sync)
        if (int r = team_join(c)) return r;
    hipLaunchKernelGGL(shmk_barrier_exchange, dim3(c->npes), dim3(SHMK_WG), 0, c->stream[0], dev_view(c), dst_off, src_off, acc_off, n,
                       rounds);
    if (int r = launched("barrier exchange")) return r;
    if (c->team_sync)
        if (int r = team_fork(c)) return r;
    return SHM_OK;
}

int shm_launch_sync_all(shm_ctx *c, int rounds, int with_quiet, uint64_t *dev_ticks)
{
    if (int r = check_ctx(c)) return r;
    if (rounds < 1 || rounds > (1 << 20)) return fail(SHM_EINVAL, "rounds outside 1..2^20");
    if (!dev_ticks) return fail(SHM_EINVAL, "null tick buffer");
    if (c->no_device) return no_device("shm_launch_sync_all");
    if (int r = drain_all_engines(c)) return r;
    if (c->team_sync)
        if (int r = team_join(c)) return r;
    hipLaunchKernelGGL(shmk_sync_all, dim3(c->npes), dim3(SHMK_WG), 0, c->stream[0], dev_view(c), rounds, with_quiet,
                       reinterpret_cast<unsigned long long *>(dev_ticks));
    if (int r = launched("sync")) return r;
    if (c->team_sync)
        if (int r = team_fork(c)) return r;
    return SHM_OK;
}

int shm_launch_broadcast(shm_ctx *c, uint64_t dst_off, uint64_t src_off, size_t n, int root, int n_wg, int path)
{
    if (int r = check_ctx(c)) return r;
    if (int r = check_pe(c, root, "root PE")) return r;
    if (int r = check_range(c, src_off, n, "source")) return r;
    if (int r = check_range(c, dst_off, n, "destination")) return r;
    if (overlaps(dst_off, src_off, n)) return fail(SHM_EINVAL, "source and destination overlap");
    if (int r = check_n_wg(n_wg)) return r;
    int use;
    if (int r = resolve_collective_path(c, SHM_COLL_BROADCAST, path, n, n_wg, &use)) return r;
    if (c->no_device) return no_device("shm_launch_broadcast");
    if (int r = drain_all_engines(c)) return r;
    if (n == 0) return team_order_only(c);
    if (c->team_sync)
        if (int r = team_join(c)) return r;
    if (use != SHM_PATH_LDST) {
        if (c->team_sync)
            if (int r = team_fork(c)) return r;
        for (int j = 0; j < c->npes; ++j) {          // one copy per destination, spread over the PE streams / engines
            const int q = (root + 1 + j) % c->npes;
            if (int r = transfer_copy(c, use, q, q, dst_off, root, src_off, n)) return r;
        }
        if (c->team_sync) {
            // the engines are not on the streams: only the host can put later work of OTHER PEs behind them
            if (use == SHM_PATH_SDMA)
                if (int r = drain_all_engines(c)) return r;
            if (int r = team_join(c)) return r;
            if (int r = team_fork(c)) return r;
        }
        return SHM_OK;
    }
    // A long block asked of a group per compute unit or more is pushed by exactly that many groups, which draw 16 KiB
    // pieces of it by ticket like fcollect's (measured, 8 PEs, root's block of 64 / 256 MiB, % of the HBM roofline:
    // 60.5 -> 78.6 and 62.5 -> 84.3; 16 MiB level at 28-29 us; 128 / 192 / 384 / 512 groups: 63 / 76 / 78 / 77 % at 256 MiB).
    uint64_t pair = 0;
    if (((dst_off | src_off) & 15) == 0 && n >= BROADCAST_TICKETS_MIN_BYTES && n_wg >= c->num_cu) {
        n_wg = c->num_cu;
        pair = ticket_pair_off(c, SHMD_TICKET_COLL);
    }
    else if (n >= (size_t(4) << 20))       // a whole number of groups per compute unit (8 MiB asked of 300 / 400 / 600 groups: 52 / 55 / 54 -> 66 / 66 / 64 %)
        n_wg = static_cast<int>(balanced_groups(c, static_cast<unsigned>(n_wg), 1));
    hipLaunchKernelGGL(shmk_broadcast, dim3(n_wg), dim3(SHMK_WG), 0, c->stream[0], dev_view(c), dst_off, src_off, n, root, pair);
    if (int r = launched("broadcast")) return r;
    if (c->team_sync)
        if (int r = team_fork(c)) return r;
    return SHM_OK;
}

int shm_launch_reduce_sum_f32(shm_ctx *c, uint64_t dst_off, uint64_t src_off, size_t nelems, int n_wg, int algo)
{
    if (int r = check_ctx(c)) return r;
    if (nelems > c->user_bytes / 4) return fail(SHM_ERANGE, "vector leaves the heap");
    if (int r = check_range(c, src_off, nelems * 4, "source")) return r;
    if (int r = check_range(c, dst_off, nelems * 4, "destination")) return r;
    if ((src_off | dst_off) & 3) return fail(SHM_EINVAL, "float32 vectors must be 4-byte aligned");
    if (overlaps(dst_off, src_off, nelems * 4)) return fail(SHM_EINVAL, "source and destination overlap");
    if (int r = check_team_grid(c, n_wg)) return r;
    if (algo != SHM_REDUCE_DUPLICATE && algo != SHM_REDUCE_SPLIT) return fail(SHM_EINVAL, "unknown reduce algorithm %d", algo);
    if (c->no_device) return no_device("shm_launch_reduce_sum_f32");
    if (int r = drain_all_engines(c)) return r;
    if (nelems == 0) return team_order_only(c);
    if (c->team_sync)
        if (int r = team_join(c)) return r;
    const shm_dev_ctx d = dev_view(c);
    const dim3 grid(n_wg, c->npes), block(SHMK_WG);
    size_t done = 0;
    if (((src_off | dst_off) & 15) == 0 && nelems >= 4) {
        const size_t nvec = nelems / 4;
        if (algo == SHM_REDUCE_SPLIT) {
            uint64_t pair = 0;
            const int groups = split_reduce_groups(c, nvec, n_wg, &pair);
            hipLaunchKernelGGL(shmk_reduce_sum_f32_vec<true>, dim3(groups, c->npes), block, 0, c->stream[0], d, dst_off, src_off, nvec, pair);
        } else
            hipLaunchKernelGGL(shmk_reduce_sum_f32_vec<false>, dim3(duplicate_reduce_groups(c, nelems * 4, n_wg), c->npes), block, 0, c->stream[0], d,
                               dst_off, src_off, nvec, uint64_t(0));
        if (int r = launched("sum-reduce")) return r;
        done = nvec * 4;
    }
    if (done < nelems) {
        const dim3 sgrid(done ? 1 : n_wg, c->npes);
        hipLaunchKernelGGL(shmk_reduce_sum_f32_scalar, sgrid, block, 0, c->stream[0], d, dst_off, src_off, done, nelems);
        if (int r = launched("sum-reduce tail")) return r;
    }
    if (c->team_sync)
        if (int r = team_fork(c)) return r;
    return SHM_OK;
}

}  // extern "C"
