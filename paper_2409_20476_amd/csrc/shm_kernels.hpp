// __global__ drivers around the device API of shm_device.hpp.  One work-group = 256 threads
// (4 wave64).  Grids are (groups per PE, PEs) so that blockIdx.y names the calling PE.
#pragma once

#include "shm_device.hpp"

#define SHMK_WG 256

typedef float shm_f32x4 __attribute__((ext_vector_type(4)));

// Split reductions walk a PE's slice on group-owned 64 KiB tiles from this many tiles per PE.
#define SHMK_OWNED_MIN_TILES 64
#define SHMK_STORE_LINE static_cast<unsigned>(SHM_STORE_LINE)       // long walks by ticket start on a destination address that is a multiple of this
#define SHMK_REDUCE_PIECES 4        // pieces per 64 KiB tile that a long split reduction draws by ticket

// ---- work-group put / get, one PE or a team of PEs in one grid ----------------------------
// PE me = me0 + blockIdx.y targets PE (me + shift) mod npes; group blockIdx.x of gridDim.x takes
// its share of the message.
__global__ __launch_bounds__(SHMK_WG) void shmk_wg_rma(shm_dev_ctx c, uint64_t dst_off, uint64_t src_off, size_t n, int me0,
                                                       int shift, int is_get)
{
    const int me = me0 + blockIdx.y;
    int pe = me + shift;
    if (pe >= c.npes) pe -= c.npes;
    if (is_get)
        shmx_getmem_parts(c, me, dst_off, src_off, n, pe, blockIdx.x, gridDim.x);
    else
        shmx_putmem_parts(c, me, dst_off, src_off, n, pe, blockIdx.x, gridDim.x);
}

// Long messages.  The dynamic LDS the host asks for is never touched: it only caps how many groups a
// CU holds at once.  What a group does before its first load counts: the kernel takes the heap as
// base address and partition stride (the library's partitions are equally spaced) instead of the
// whole device view -- one scalar load of the arguments, no table look-up.
// ticket_pair_off == 0: group-owned tiles, group g of gridDim.x taking tiles g, g + gridDim.x, ...
// (offsets 16-byte aligned).
// ticket_pair_off != 0: the offset, in every partition, of a counter pair that reads zero: the
// gridDim.x groups of a PE draw half-tile pieces by ticket from their own PE's pair (shm_copy_tiles_ticketed;
// every group starts on the piece of its own number) and the last one through sets the pair back; ways: see below.
__global__ __launch_bounds__(SHMK_WG) void shmk_wg_rma_tiles(char *base, uint64_t stride, uint64_t dst_off, uint64_t src_off, size_t n,
                                                             int npes, int me0, int shift, int is_get, uint64_t ticket_pair_off,
                                                             unsigned ways)
{
    const int me = me0 + blockIdx.y;
    int pe = me + shift;
    if (pe >= npes) pe -= npes;
    // one copy of the walk for both directions: only the two addresses differ
    char *d = base + static_cast<uint64_t>(is_get ? me : pe) * stride + dst_off;
    const char *s = base + static_cast<uint64_t>(is_get ? pe : me) * stride + src_off;
    // Either walk starts where the destination reaches a multiple of SHMK_STORE_LINE bytes; the bytes
    // before it are moved by the last group (on tiles: whole vectors, the addresses being 16-byte aligned).
    // Stores that straddle lines cost far more than loads that do (8 PEs x 128 MiB by ticket; destination
    // alone 16 bytes past a boundary: 75.4 % of the HBM roofline walking from there, 81.4 % from the next
    // boundary; both 16 bytes past: 73.1 -> 83.7 %; neither: 83.9 %).
    size_t head = (SHMK_STORE_LINE - (reinterpret_cast<uintptr_t>(d) & (SHMK_STORE_LINE - 1))) & (SHMK_STORE_LINE - 1);
    if (head > n) head = n;
    if (blockIdx.x == gridDim.x - 1) {
        if (ticket_pair_off == 0) {
            if (threadIdx.x < head / 16)
                shm_st16(reinterpret_cast<shm_u32x4 *>(d) + threadIdx.x, shm_ld16(reinterpret_cast<const shm_u32x4 *>(s) + threadIdx.x));
        } else {
            for (size_t i = threadIdx.x; i < head; i += SHMK_WG) d[i] = s[i];
        }
    }
    d += head, s += head, n -= head;
    if (ticket_pair_off == 0) {
        shmx_copy_tiles_wg<SHMK_WG / 64>(d, s, n, blockIdx.x, gridDim.x);
        return;
    }
    // By ticket, at any byte addresses: a source that is now not on a 16-byte boundary is read as the
    // aligned words around each vector; the bytes after the last whole vector are moved by the first group.
    const size_t body = n & ~static_cast<size_t>(15);
    if (blockIdx.x == 0)
        for (size_t i = body + threadIdx.x; i < n; i += SHMK_WG) d[i] = s[i];
    // ways > 1 (a divisor of gridDim.x): the message is walked as that many runs of whole tiles, each by
    // its share of the groups on a counter pair of its own, SHMD_TICKET_WAY_BYTES further on
    const unsigned groups = gridDim.x / ways, way = blockIdx.x / groups, part = blockIdx.x - way * groups;
    const size_t tiles = body >> 16, lo = (tiles * way / ways) << 16, hi = way + 1 == ways ? body : (tiles * (way + 1) / ways) << 16;
    unsigned long long *pair = reinterpret_cast<unsigned long long *>(base + static_cast<uint64_t>(me) * stride + ticket_pair_off +
                                                                      static_cast<uint64_t>(way) * SHMD_TICKET_WAY_BYTES);
    shm_copy_tiles_ticketed_any<2, SHMK_WG / 64>(d + lo, s + lo, hi - lo, part, pair, 0, groups);
    if (threadIdx.x == 0) shm_tickets_done(pair, groups);
}

// One-direction ceilings of the memory system with the access forms of the long-message put: the
// team grid, but every byte is only read (KIND 0: 16-byte nontemporal loads of the source on the
// calling PE, folded into a word that is stored only if it equals `magic`, which keeps the loads
// alive) or only written (KIND 1: 16-byte nontemporal stores of a lane-dependent pattern to the
// destination on the target PE).
// FORM 0: group-owned 64 KiB tiles.  FORM 1: a front -- the PE's groups sweep the block together,
// every group one 4 KiB piece of a front of gridDim.x pieces that moves through the block.  FORM 2:
// half-tile pieces by ticket, exactly the walk of the long put (ticket_pair_off as there).
template <int KIND, int FORM>
__global__ __launch_bounds__(SHMK_WG) void shmk_stream_probe(shm_dev_ctx c, uint64_t dst_off, uint64_t src_off, size_t n, int shift,
                                                             uint32_t magic, uint64_t ticket_pair_off)
{
    const int me = blockIdx.y;
    int pe = me + shift;
    if (pe >= c.npes) pe -= c.npes;
    const shm_u32x4 *s = reinterpret_cast<const shm_u32x4 *>(shm_ptr(c, src_off, me));
    shm_u32x4 *d = reinterpret_cast<shm_u32x4 *>(shm_ptr(c, dst_off, pe));
    constexpr size_t rowv = 2048, tilev = 2 * rowv;
    const size_t ntiles = (n >> 4) / tilev;                 // whole tiles only: n is a multiple of 64 KiB
    const unsigned wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    uint32_t fold = 0;
    shm_u32x4 pattern;
    pattern.x = threadIdx.x, pattern.y = blockIdx.x, pattern.z = magic, pattern.w = static_cast<uint32_t>(me);
    if (FORM == 2) {
        unsigned long long *pair = reinterpret_cast<unsigned long long *>(shm_ptr(c, ticket_pair_off, me));
        char *db = reinterpret_cast<char *>(d);
        const char *sb = reinterpret_cast<const char *>(s);
        if (KIND == 0) {
            shm_walk_read ops;
            shm_walk_tiles_ticketed<2, SHMK_WG / 64, 2>(ops, db, sb, n, blockIdx.x, pair, 0, gridDim.x);
            fold = ops.fold;
        } else {
            shm_walk_write ops{pattern};
            shm_walk_tiles_ticketed<2, SHMK_WG / 64, 2>(ops, db, sb, n, blockIdx.x, pair, 0, gridDim.x);
        }
        if (threadIdx.x == 0) shm_tickets_done(pair, gridDim.x);
        if (KIND == 0 && fold == magic && n == 1) d[0].x = fold;
        return;
    }
    if (FORM == 1) {
        const size_t nvec = n >> 4, step = static_cast<size_t>(gridDim.x) * SHMK_WG;
        size_t i = static_cast<size_t>(blockIdx.x) * SHMK_WG + threadIdx.x;
        for (; i + 3 * step < nvec; i += 4 * step) {           // four steps of the front in flight per lane
            if (KIND == 0) {
                shm_u32x4 r[4];
#pragma unroll
                for (int u = 0; u < 4; ++u) r[u] = shm_ld16(s + i + u * step);
#pragma unroll
                for (int u = 0; u < 4; ++u) fold ^= r[u].x ^ r[u].y ^ r[u].z ^ r[u].w;
            } else {
#pragma unroll
                for (int u = 0; u < 4; ++u) shm_st16(d + i + u * step, pattern);
            }
        }
        for (; i < nvec; i += step) {
            if (KIND == 0) {
                const shm_u32x4 r0 = shm_ld16(s + i);
                fold ^= r0.x ^ r0.y ^ r0.z ^ r0.w;
            } else {
                shm_st16(d + i, pattern);
            }
        }
        if (KIND == 0 && fold == magic && n == 1) d[0].x = fold;
        return;
    }
    for (size_t t = blockIdx.x; t < ntiles; t += gridDim.x) {
#pragma unroll
        for (unsigned cc = 0; cc < 8; ++cc) {
            const size_t i = t * tilev + static_cast<size_t>(wave * 8 + cc) * 64 + lane;
            if (KIND == 0) {
                const shm_u32x4 r0 = shm_ld16(s + i), r1 = shm_ld16(s + i + rowv);
                fold ^= r0.x ^ r0.y ^ r0.z ^ r0.w ^ r1.x ^ r1.y ^ r1.z ^ r1.w;
            } else {
                shm_st16(d + i, pattern);
                shm_st16(d + i + rowv, pattern);
            }
        }
    }
    if (KIND == 0 && fold == magic && n == 1) d[0].x = fold;       // never true for a launch the host accepts
}

// The same put repeated `reps` times inside one kernel, each followed by the group's quiet, with the
// device clock read before the first and after the last: the cost of a put issued from a running
// kernel, free of any launch overhead.  ticks[0] = earliest start, ticks[1] = latest end over the groups
// that have a share of the message.
// FORM 0: the general dealing; 1: long message on group-owned tiles (the launcher's choice, as for an
// untimed put); 2: the same tiles drawn by ticket, repetition r from the r-th ticket word of this PE's
// tail, which reads 0.  One kernel per form: the loop of a short put stays a few hundred instructions.
template <int FORM>
__global__ __launch_bounds__(SHMK_WG) void shmk_wg_put_timed(shm_dev_ctx c, uint64_t dst_off, uint64_t src_off, size_t n, int me, int pe,
                                                             int reps, unsigned long long *ticks)
{
    // groups without a share have nothing to complete
    const bool mine = FORM ? blockIdx.x < (n + 65535) / 65536 : shm_deal_has_share<8>(n, blockIdx.x, gridDim.x, SHMK_WG, SHM_MIN_SHARE_BYTES);
    const bool bulk = FORM || !shm_put_stores_through(n, gridDim.x, SHM_MIN_SHARE_BYTES);
    [[maybe_unused]] unsigned long long *tickets =
        reinterpret_cast<unsigned long long *>(shm_ptr(c, c.internal_off + SHMD_INTERNAL_TICKETS, me));
    const unsigned long long t0 = wall_clock64();
    for (int r = 0; r < reps; ++r) {
        if constexpr (FORM == 2)
            shmx_putmem_tickets<SHMK_WG / 64>(c, me, dst_off, src_off, n, pe, blockIdx.x, tickets + r, 0, gridDim.x);
        else if constexpr (FORM == 1)
            shmx_putmem_tiles<SHMK_WG / 64>(c, me, dst_off, src_off, n, pe, blockIdx.x, gridDim.x);
        else
            shmx_putmem_parts(c, me, dst_off, src_off, n, pe, blockIdx.x, gridDim.x, SHM_MIN_SHARE_BYTES);
        if (mine) shmx_quiet_wg(c, bulk);
    }
    const unsigned long long t1 = wall_clock64();
    // Only the groups that moved bytes report: a group without a share returns from every put at
    // once, and when the dispatcher gets round to starting it is launch overhead, not part of the put.
    if (threadIdx.x == 0 && mine) {
        atomicMin(&ticks[0], t0);
        atomicMax(&ticks[1], t1);
    }
}

// Device-initiated put or get, `reps` times, by gridDim.x groups (of 64..1024 threads: the paper
// varies the work-items per work-group) that each own a contiguous 256-byte-aligned share of the
// message.  mode 0: loads/stores (put: + group quiet); 1: host-started copy engine, blocking;
// 2: cutover on the share size; 3: non-blocking engine transfer (put_nbi / get_nbi), offload quiet
// after each; 4: engine for all but the first `cover` bytes of the share, loads/stores for those,
// then both quiets; 5: non-blocking engine transfer and no quiet at all inside the kernel -- the
// transfer is complete after the host's quiet for this PE.  consume_off (get only, else UINT64_MAX): before the first get the group copies
// its share of the destination to consume_off -- which pulls the old bytes into the caches -- and
// after every get it copies the share again, so the copy shows what a thread of the group reads.
constexpr uint64_t SHMK_NO_CONSUME = ~0ull;

// One kernel per mode and direction (compile-time): what a repetition runs through stays short, which
// is worth a quarter of a small put's time against one kernel that branches on the mode.
template <int MODE, bool IS_GET>
__global__ __launch_bounds__(1024) void shmk_rma_device_initiated(shm_dev_ctx c, uint64_t dst_off, uint64_t src_off, size_t n, int me,
                                                                     int pe, size_t cutover, size_t cover, uint64_t consume_off, int reps,
                                                                     unsigned long long *ticks)
{
    constexpr int mode = MODE;
    constexpr bool is_get = IS_GET;
    size_t per = (n + gridDim.x - 1) / gridDim.x;
    per = (per + 255) & ~static_cast<size_t>(255);
    const size_t lo = min(n, blockIdx.x * per), len = min(n, lo + per) - lo;
    const uint64_t d = dst_off + lo, s = src_off + lo;
    const bool consume = is_get && consume_off != SHMK_NO_CONSUME;
    if (consume) shmx_putmem_wg(c, me, consume_off + lo, d, len, me);
    const unsigned long long t0 = wall_clock64();
    for (int r = 0; r < reps; ++r) {
        if constexpr (mode == 0) {
            if (is_get) {
                shmx_getmem_wg(c, me, d, s, len, pe);
            } else {
                shmx_putmem_wg(c, me, d, s, len, pe);
                if (len) shmx_quiet_wg(c, !shm_put_stores_through(len));
            }
        } else if constexpr (mode == 1) {
            if (is_get)
                shmx_getmem_offload_wg(c, me, d, s, len, pe, true);
            else
                shmx_putmem_offload_wg(c, me, d, s, len, pe, true);
        } else if constexpr (mode == 2) {
            const bool engine = c.off.ring != nullptr && len >= shm_resolve_cutover(cutover);
            if (is_get) {
                shmx_getmem_auto_wg(c, me, d, s, len, pe, cutover);
            } else {
                shmx_putmem_auto_wg(c, me, d, s, len, pe, cutover);
                if (!engine && len) shmx_quiet_wg(c, !shm_put_stores_through(len));
            }
        } else if constexpr (mode == 3) {
            if (is_get)
                shmx_getmem_offload_wg(c, me, d, s, len, pe, false);
            else
                shmx_putmem_offload_wg(c, me, d, s, len, pe, false);
            shmx_quiet_offload_wg(c, me);
        } else if constexpr (mode == 5) {
            if (is_get)
                shmx_getmem_offload_wg(c, me, d, s, len, pe, false);
            else
                shmx_putmem_offload_wg(c, me, d, s, len, pe, false);
        } else {
            shmx_rma_covered_wg(c, me, d, s, len, pe, cover, is_get);
            if (!is_get && len) shmx_quiet_wg(c);
            shmx_quiet_offload_wg(c, me);
        }
        if (consume) shmx_putmem_wg(c, me, consume_off + lo, d, len, me);
    }
    const unsigned long long t1 = wall_clock64();
    if (ticks != nullptr && threadIdx.x == 0) {
        atomicMin(&ticks[0], t0);
        atomicMax(&ticks[1], t1);
    }
}

// One work-item of the whole device calls the single-thread put or get `reps` times (the paper's
// first experiment: bandwidth of ishmem_put / ishmem_get issued by one thread), quiet after each put.
__global__ __launch_bounds__(64) void shmk_thread_rma(shm_dev_ctx c, uint64_t dst_off, uint64_t src_off, size_t n, int me, int pe,
                                                      int is_get, int reps, unsigned long long *ticks)
{
    if (threadIdx.x != 0 || blockIdx.x != 0) return;
    const unsigned long long t0 = wall_clock64();
    for (int r = 0; r < reps; ++r) {
        if (is_get) {
            shm_getmem<32>(c, me, dst_off, src_off, n, pe);
            __builtin_amdgcn_s_waitcnt(0);          // a get returns with the bytes in place
        } else {
            shm_putmem<32>(c, me, dst_off, src_off, n, pe);
            shm_quiet();
        }
    }
    const unsigned long long t1 = wall_clock64();
    if (ticks != nullptr) {
        atomicMin(&ticks[0], t0);
        atomicMax(&ticks[1], t1);
    }
}

// Scalar p / g, one element per work-item (grid-stride).  is_get == 0: work-item i reads element i
// of its own PE's source and p's it to the target PE's destination.  is_get != 0: it g's element i
// of the target PE's source and stores it to its own PE's destination.
template <typename T>
__global__ __launch_bounds__(SHMK_WG) void shmk_scalar_pg(shm_dev_ctx c, uint64_t dst_off, uint64_t src_off, size_t nelems, int me,
                                                          int pe, int is_get)
{
    const size_t step = static_cast<size_t>(gridDim.x) * SHMK_WG;
    for (size_t i = static_cast<size_t>(blockIdx.x) * SHMK_WG + threadIdx.x; i < nelems; i += step) {
        if (is_get)
            reinterpret_cast<T *>(shm_ptr(c, dst_off, me))[i] = shm_g<T>(c, src_off + i * sizeof(T), pe);
        else
            shm_p<T>(c, dst_off + i * sizeof(T), reinterpret_cast<const T *>(shm_ptr(c, src_off, me))[i], pe);
    }
}

// Strided put/get.  single != 0: one work-item does the whole transfer (ishmem_iput / ishmem_iget);
// otherwise the gridDim.x groups share the elements (the work-group forms).
__global__ __launch_bounds__(SHMK_WG) void shmk_strided(shm_dev_ctx c, uint64_t dst_off, uint64_t src_off, size_t dst_stride,
                                                        size_t src_stride, size_t nelems, uint32_t elem_bytes, int me, int pe,
                                                        int is_get, int single)
{
    if (single) {
        if (threadIdx.x != 0 || blockIdx.x != 0) return;
        if (is_get)
            shm_iget(c, me, dst_off, src_off, dst_stride, src_stride, nelems, elem_bytes, pe);
        else
            shm_iput(c, me, dst_off, src_off, dst_stride, src_stride, nelems, elem_bytes, pe);
        return;
    }
    if (is_get)
        shmx_iget_parts(c, me, dst_off, src_off, dst_stride, src_stride, nelems, elem_bytes, pe, blockIdx.x, gridDim.x);
    else
        shmx_iput_parts(c, me, dst_off, src_off, dst_stride, src_stride, nelems, elem_bytes, pe, blockIdx.x, gridDim.x);
}

// Ring micro-benchmark: wave 0 of every group sends `reps` empty requests.  blocking: waits for
// each answer (round trips).  Otherwise fire-and-forget, one quiet with an answer at the end (rate).
__global__ __launch_bounds__(SHMK_WG) void shmk_offload_nop(shm_dev_ctx c, int me, int reps, int blocking, unsigned long long *ticks)
{
    const unsigned long long t0 = wall_clock64();
    if (threadIdx.x < 64) {
        for (int r = 0; r < reps; ++r) {
            const uint64_t ticket = shm_offload_send(c, SHMD_OFFLOAD_NOP, me, 0, 0, 0, blocking != 0);
            if (blocking) shm_offload_wait(c, ticket);
        }
        if (!blocking) shm_offload_wait(c, shm_offload_send(c, SHMD_OFFLOAD_NOP, me, 0, 0, 0, true));
    }
    __syncthreads();
    const unsigned long long t1 = wall_clock64();
    if (threadIdx.x == 0) {
        atomicMin(&ticks[0], t0);
        atomicMax(&ticks[1], t1);
    }
}

__global__ __launch_bounds__(SHMK_WG) void shmk_wg_put_signal(shm_dev_ctx c, int me, int pe, uint64_t dst_off, uint64_t src_off,
                                                              size_t n, uint64_t sig_off, uint64_t sig_val, int sig_op,
                                                              uint64_t *arrive)
{
    shmx_putmem_signal_parts(c, me, dst_off, src_off, n, sig_off, sig_val, sig_op, pe, arrive, blockIdx.x, gridDim.x);
}

__global__ __launch_bounds__(SHMK_WG) void shmk_signal_wait(shm_dev_ctx c, int me, uint64_t sig_off, int cmp, uint64_t val,
                                                            uint64_t *out)
{
    const uint64_t v = shmx_signal_wait_until_wg(c, me, sig_off, cmp, val);
    if (out != nullptr && threadIdx.x == 0) *out = v;
}

// ---- point-to-point synchronisation: wait_until / test and their all / any / some forms ------
// One thread of PE `me`.  kind: 0 wait, 1 wait_all, 2 wait_any, 3 wait_some, 4 test, 5 test_all,
// 6 test_any, 7 test_some.  out[0] = the call's result (the satisfying value for wait, 1/0 for the
// tests that answer yes or no, the index for any -- UINT64_MAX if there is none --, the count for
// some); for the some forms out[1 ..] = the indices.
__global__ __launch_bounds__(64) void shmk_sync_set(shm_dev_ctx c, int me, uint64_t off, size_t n, const int *status, int kind, int cmp,
                                                    long long val, unsigned long long *out)
{
    if (threadIdx.x != 0 || blockIdx.x != 0) return;
    size_t *indices = reinterpret_cast<size_t *>(out + 1);
    unsigned long long r = 0;
    switch (kind) {
    case 0: r = static_cast<unsigned long long>(shm_wait_until(c, me, off, cmp, val)); break;
    case 1: shm_wait_until_all(c, me, off, n, status, cmp, val); r = 1; break;
    case 2: r = shm_wait_until_any(c, me, off, n, status, cmp, val); break;
    case 3: r = shm_wait_until_some(c, me, off, n, indices, status, cmp, val); break;
    case 4: r = shm_test(c, me, off, cmp, val) ? 1 : 0; break;
    case 5: r = shm_test_all(c, me, off, n, status, cmp, val) ? 1 : 0; break;
    case 6: r = shm_test_any(c, me, off, n, status, cmp, val); break;
    default: r = shm_test_some(c, me, off, n, indices, status, cmp, val); break;
    }
    out[0] = r;
}

// ---- one atomic by one work-item ---------------------------------------------------------
__global__ void shmk_amo(shm_dev_ctx c, int pe, uint64_t off, int op, int64_t operand, int64_t cond, int64_t *out)
{
    if (threadIdx.x != 0 || blockIdx.x != 0) return;
    int64_t r = 0;
    switch (op) {
    case 0: r = shm_atomic_fetch(c, off, pe); break;
    case 1: shm_atomic_set(c, off, operand, pe); break;
    case 2: r = shm_atomic_swap(c, off, operand, pe); break;
    case 3: r = shm_atomic_compare_swap(c, off, cond, operand, pe); break;
    case 4: r = shm_atomic_fetch_add(c, off, operand, pe); break;
    case 5: shm_atomic_add(c, off, operand, pe); break;
    case 6: r = shm_atomic_fetch_inc(c, off, pe); break;
    default: shm_atomic_inc(c, off, pe); break;
    }
    if (out != nullptr) *out = r;
}

// ---- configuration 1: put, quiet, flag / wait, get back -----------------------------------
__global__ __launch_bounds__(SHMK_WG) void shmk_ping_producer(shm_dev_ctx c, uint64_t data_off, size_t n, uint64_t flag_off)
{
    shmx_putmem_wg(c, 0, data_off, data_off, n, 1);
    shmx_quiet_wg();                                                                  // orders the payload before the flag
    shmx_putmem_signal_wg(c, 0, data_off, data_off, 0, flag_off, 1, SHMD_SIGNAL_SET, 1);  // zero-byte payload, flag := 1
}

__global__ __launch_bounds__(SHMK_WG) void shmk_ping_consumer(shm_dev_ctx c, uint64_t data_off, uint64_t back_off, size_t n,
                                                              uint64_t flag_off)
{
    shmx_signal_wait_until_wg(c, 1, flag_off, SHMD_CMP_EQ, 1);
    shmx_getmem_wg(c, 1, back_off, data_off, n, 0);
}

// ---- the sub-group (wave) forms in one program --------------------------------------------------
// Blocks [0, G) are producers of PE `me`, blocks [G, 2G) consumers of PE `pe`; wave w (4 per group)
// owns the w-th 16-byte-rounded share of the message.  Producer wave: wave put, fence, lane 0 sets
// flag w on pe.  Consumer wave: lane 0 waits for flag w (bounded) and records what signal_fetch
// returns; the wave then gets its share from pe's own destination into `back`.  Producers come first
// in the grid and never wait; the host refuses a grid that cannot be resident as a whole.
__global__ __launch_bounds__(SHMK_WG) void shmk_wave_exchange(shm_dev_ctx c, uint64_t dst_off, uint64_t src_off, uint64_t back_off,
                                                              size_t n, int n_waves, uint64_t flag_off, uint64_t out_off, int me, int pe)
{
    const int groups = (n_waves + 3) / 4;
    const bool producer = static_cast<int>(blockIdx.x) < groups;
    const int w = (producer ? blockIdx.x : blockIdx.x - groups) * 4 + (threadIdx.x >> 6);
    if (w >= n_waves) return;
    size_t per = (n + n_waves - 1) / n_waves;
    per = (per + 15) & ~static_cast<size_t>(15);
    const size_t lo = min(n, static_cast<size_t>(w) * per), len = min(n, lo + per) - lo;
    const uint64_t flag = flag_off + 8ull * w;
    if (producer) {
        shmx_putmem_wave(c, me, dst_off + lo, src_off + lo, len, pe);
        shm_fence();                                            // the share is delivered before the flag
        if (__lane_id() == 0) shm_atomic_set(c, flag, 1, pe);
        return;
    }
    if (__lane_id() == 0) {
        (void)shm_signal_wait_until(c, pe, flag, SHMD_CMP_EQ, 1);
        *reinterpret_cast<uint64_t *>(shm_ptr(c, out_off + 8ull * w, pe)) = shm_signal_fetch(c, pe, flag);
    }
    shmx_getmem_wave(c, pe, back_off + lo, dst_off + lo, len, pe);
}

// ---- configuration 3: pipelined ring --------------------------------------------------------
// Blocks [0, npes*n_prod) are producers, the rest consumers; PE = index mod npes so that the
// groups of one PE are spread over the dispatch order.  Producers never wait, and they come first
// in the grid, so consumers cannot starve them.
#define SHMK_RING_VPT 8      // 16-byte vectors (8 bf16) per consumer thread held in registers

// LANES: one signal word per producer/consumer group pair (compile-time, so that each form carries
// only its own code and registers: both fit 128 VGPRs, four groups per compute unit).
// DEEP: for producer shares of more than 32 KiB and up to 128 KiB per chunk (fewer than 32 producer
// groups per PE at 1 MiB chunks), which do not fit the two-half form's registers: the whole group
// walks its share in blocks of 64 KiB -- 16 vectors per thread -- and keeps TWO blocks in registers,
// loading block s+1 while the stores of block s are on their way, 128 KiB in flight per group; the
// chunk is signalled after the acknowledgements of its last block.  That needs 137 registers, so
// this form is a kernel of its own (three groups per compute unit instead of four).  Measured, 8 PEs x
// 64 chunks of 1 MiB: 8 producer groups per PE 0.60 -> 0.55 ms, 16 groups 0.415 -> 0.366 ms (32 groups,
// two-half form: 0.26 ms): a step still lasts as long as its slower half, the loads or the stores'
// acknowledgements, and few groups mean few steps in flight.
#define SHMK_RING_DEEP_VPT 16
template <int LANES, int DEEP = 0>
__global__ __launch_bounds__(SHMK_WG, DEEP ? 2 : 4) void shmk_ring(shm_dev_ctx c, uint64_t src_off, uint64_t slot_off, uint64_t sig_off,
                                                        uint64_t acc_off, size_t chunk_bytes, int n_chunks, int n_prod, int n_cons,
                                                        uint64_t *arrive_pe0, uint64_t arrive_pe_stride)
{
    // arrival counters, one per chunk: PE p's are at arrive_pe0 + p * arrive_pe_stride (in words)
    constexpr bool lanes = LANES != 0;
    const int npes = c.npes;
    const int b = blockIdx.x;
    const size_t nvec = chunk_bytes >> 4;
    const size_t per = (nvec + n_cons - 1) / n_cons;           // host guarantees per <= SHMK_WG * SHMK_RING_VPT
    if (b < npes * n_prod) {
        const int me = b % npes, part = b / npes;
        int pe = me + 1;
        if (pe >= npes) pe = 0;
        const size_t pper = lanes ? per : (nvec + n_prod - 1) / n_prod;     // this producer's share of a chunk, in vectors
        if constexpr (DEEP != 0) {
            constexpr int J = SHMK_RING_DEEP_VPT;
            constexpr uint32_t BLOCK = SHMK_WG * J;                        // vectors per block
            const size_t lo = min(nvec, part * pper), hi = min(nvec, lo + pper);
            const bool any = hi > lo;
            const uint32_t last = any ? static_cast<uint32_t>(hi - 1 - lo) : 0;
            const int nsub = static_cast<int>((pper + BLOCK - 1) / BLOCK);  // blocks per chunk; the host allows up to 2
            const shm_u32x4 *s = reinterpret_cast<const shm_u32x4 *>(shm_ptr(c, src_off, me)) + lo;
            shm_u32x4 *d = reinterpret_cast<shm_u32x4 *>(shm_ptr(c, slot_off, pe)) + lo;
            uint64_t *sig = reinterpret_cast<uint64_t *>(shm_ptr(c, sig_off, pe));
            uint64_t *arrive = arrive_pe0 + static_cast<uint64_t>(me) * arrive_pe_stride;
            // vector of the share that thread t touches in block `sub`, access j; past the share: its last vector again
            auto v = [&](int sub, int j) { return min(last, static_cast<uint32_t>(sub) * BLOCK + threadIdx.x + static_cast<uint32_t>(j) * SHMK_WG); };
            const int steps = n_chunks * nsub;
            shm_u32x4 a[J], b[J];
            auto load = [&](shm_u32x4 (&r)[J], int step) {
                const size_t at = static_cast<size_t>(step / nsub) * nvec;
                const int sub = step % nsub;
#pragma unroll
                for (int j = 0; j < J; ++j) r[j] = shm_ld16(s + at + v(sub, j));
            };
            auto store_and_signal = [&](shm_u32x4 (&r)[J], int step) {
                const int k = step / nsub, sub = step % nsub;
                if (any) {
#pragma unroll
                    for (int j = 0; j < J; ++j) shm_st16<SHM_ST_THROUGH>(d + static_cast<size_t>(k) * nvec + v(sub, j), r[j]);
                }
                asm volatile("s_waitcnt vmcnt(0)" ::: "memory");           // this wave's stores are performed at agent scope
                __syncthreads();
                if (sub == nsub - 1 && threadIdx.x == 0) {
                    const uint64_t old = __hip_atomic_fetch_add(arrive + k, 1ull, SHMD_ARRIVE_ORDER, __HIP_MEMORY_SCOPE_AGENT);
                    if (old == static_cast<uint64_t>(n_prod) - 1) {
                        __hip_atomic_store(arrive + k, 0ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                        __hip_atomic_fetch_add(sig, 1ull, SHMD_SIGNAL_ORDER, __HIP_MEMORY_SCOPE_AGENT);
                    }
                }
            };
            if (any) load(a, 0);
            for (int step = 0; step < steps; step += 2) {
                if (any && step + 1 < steps) load(b, step + 1);
                store_and_signal(a, step);
                if (step + 1 < steps) {
                    if (any && step + 2 < steps) load(a, step + 2);
                    store_and_signal(b, step + 1);
                }
            }
            return;
        } else
        if (pper <= static_cast<size_t>(SHMK_WG) * SHMK_RING_VPT) {
            // The share fits the group's registers.  A put_signal per chunk is a chain of two
            // memory latencies (loads, then the stores' acknowledgements), so the group works as two
            // halves that alternate: while one half stores chunk k and waits for the
            // acknowledgements, the other half already loads chunk k+1.  The barrier that ends step
            // k collects the acknowledgements of chunk k, and only then is chunk k signalled: the
            // order of a put_signal per chunk, in half the time.  With lanes the group adds 1 to its
            // own signal word; with one counter per PE it arrives on the chunk's arrival counter and
            // the group whose arrival completes the chunk adds 1 to the signal (and resets the
            // counter) -- done by the first thread of the half that loads in this step, whose wait
            // for the counter's old value overlaps its own loads.
            // Vector indices past the share are clamped to its last vector (that vector is then
            // moved more than once, with the same bytes), which keeps the loop free of predicates.
            const size_t lo = min(nvec, part * pper), hi = min(nvec, lo + pper);
            constexpr int HALF = SHMK_WG / 2, J = 2 * SHMK_RING_VPT;      // HALF * J = SHMK_WG * SHMK_RING_VPT vectors
            const int half = threadIdx.x / HALF, t = threadIdx.x % HALF;
            const shm_u32x4 *s = reinterpret_cast<const shm_u32x4 *>(shm_ptr(c, src_off, me));
            shm_u32x4 *d = reinterpret_cast<shm_u32x4 *>(shm_ptr(c, slot_off, pe));
            uint64_t *sig = reinterpret_cast<uint64_t *>(shm_ptr(c, sig_off + (lanes ? 8ull * part : 0ull), pe));
            uint64_t *arrive = arrive_pe0 + static_cast<uint64_t>(me) * arrive_pe_stride;
            const bool any = hi > lo;
            const uint32_t last = any ? static_cast<uint32_t>(hi - 1 - lo) : 0;      // a share has at most 2048 vectors
            s += lo, d += lo;
            auto v = [&](int j) { return min(last, static_cast<uint32_t>(t + j * HALF)); };
            shm_u32x4 a[J];
            if (any && half == 0) {
#pragma unroll
                for (int j = 0; j < J; ++j) a[j] = shm_ld16(s + v(j));
            }
            for (int k = 0; k < n_chunks; ++k) {
                if (any) {
                    if ((k & 1) == half) {
#pragma unroll
                        for (int j = 0; j < J; ++j) shm_st16<SHM_ST_THROUGH>(d + k * nvec + v(j), a[j]);
                        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");  // this wave's share of chunk k is performed at agent scope
                    } else if (k + 1 < n_chunks) {
#pragma unroll
                        for (int j = 0; j < J; ++j) a[j] = shm_ld16(s + (k + 1) * nvec + v(j));
                    }
                }
                __syncthreads();
                if (lanes) {
                    if (threadIdx.x == 0) __hip_atomic_fetch_add(sig, 1ull, SHMD_SIGNAL_ORDER, __HIP_MEMORY_SCOPE_AGENT);
                } else if (static_cast<int>(threadIdx.x) == ((k & 1) ? 0 : HALF)) {
                    const uint64_t old = __hip_atomic_fetch_add(arrive + k, 1ull, SHMD_ARRIVE_ORDER, __HIP_MEMORY_SCOPE_AGENT);
                    if (old == static_cast<uint64_t>(n_prod) - 1) {
                        __hip_atomic_store(arrive + k, 0ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                        __hip_atomic_fetch_add(sig, 1ull, SHMD_SIGNAL_ORDER, __HIP_MEMORY_SCOPE_AGENT);
                    }
                }
            }
            return;
        }
        // Larger shares (more than 128 KiB per chunk, or a grid too large for the DEEP form's
        // registers): one put_signal per chunk by all producer groups together.
        uint64_t *arrive = arrive_pe0 + static_cast<uint64_t>(me) * arrive_pe_stride;
        for (int k = 0; k < n_chunks; ++k)
            shmx_putmem_signal_parts(c, me, slot_off + k * chunk_bytes, src_off + k * chunk_bytes, chunk_bytes, sig_off, 1,
                                     SHMD_SIGNAL_ADD, pe, arrive + k, part, n_prod);
        return;
    }
    const int cb = b - npes * n_prod;
    const int me = cb % npes, part = cb / npes;
    const size_t lo = min(nvec, part * per), hi = min(nvec, lo + per);
    const uint64_t my_sig = sig_off + (lanes ? 8ull * part : 0ull);
    float acc[SHMK_RING_VPT][8];
#pragma unroll
    for (int j = 0; j < SHMK_RING_VPT; ++j)
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[j][e] = 0.0f;
    // Chunk k may be read once the signal counts k+1.  The leader asks for the signal's value for
    // chunk k+1 BEFORE the group loads chunk k, so that the answer travels while the data does; only
    // if it was not yet there does the leader poll.  Leader's acquire, then the barrier extends it.
    // Vector indices past the share are clamped (their sums are computed and never written).
    uint64_t *sigp = reinterpret_cast<uint64_t *>(shm_ptr(c, my_sig, me));
    const uint32_t last = hi > lo ? static_cast<uint32_t>(hi - 1 - lo) : 0;
    auto vi = [&](int j) { return lo + min(last, static_cast<uint32_t>(threadIdx.x + j * SHMK_WG)); };
    if (threadIdx.x == 0) (void)shm_signal_wait_until(c, me, my_sig, SHMD_CMP_GE, 1);
    __syncthreads();
    for (int k = 0; k < n_chunks; ++k) {
        const bool more = k + 1 < n_chunks;
        uint64_t early = 0;
        if (more && threadIdx.x == 0) early = __hip_atomic_load(sigp, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if (hi > lo) {
            const shm_u32x4 *slot = reinterpret_cast<const shm_u32x4 *>(shm_ptr(c, slot_off + k * chunk_bytes, me));
            shm_u32x4 w[SHMK_RING_VPT];
#pragma unroll
            for (int j = 0; j < SHMK_RING_VPT; ++j) w[j] = shm_ld16(slot + vi(j));
#pragma unroll
            for (int j = 0; j < SHMK_RING_VPT; ++j) {
                const uint32_t ws[4] = {w[j].x, w[j].y, w[j].z, w[j].w};
#pragma unroll
                for (int q = 0; q < 4; ++q) {      // bf16 -> f32 is a 16-bit left shift: exact
                    acc[j][2 * q] += __uint_as_float(ws[q] << 16);
                    acc[j][2 * q + 1] += __uint_as_float(ws[q] & 0xffff0000u);
                }
            }
        }
        if (more) {
            if (threadIdx.x == 0) {
                if (early >= static_cast<uint64_t>(k) + 2)
                    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
                else
                    (void)shm_signal_wait_until(c, me, my_sig, SHMD_CMP_GE, static_cast<uint64_t>(k) + 2);
            }
            __syncthreads();
        }
    }
    shm_u32x4 *out = reinterpret_cast<shm_u32x4 *>(shm_ptr(c, acc_off, me));
#pragma unroll
    for (int j = 0; j < SHMK_RING_VPT; ++j) {
        const size_t v = lo + threadIdx.x + static_cast<size_t>(j) * SHMK_WG;
        if (v < hi) {
            shm_u32x4 a, bq;
            a.x = __float_as_uint(acc[j][0]), a.y = __float_as_uint(acc[j][1]);
            a.z = __float_as_uint(acc[j][2]), a.w = __float_as_uint(acc[j][3]);
            bq.x = __float_as_uint(acc[j][4]), bq.y = __float_as_uint(acc[j][5]);
            bq.z = __float_as_uint(acc[j][6]), bq.w = __float_as_uint(acc[j][7]);
            out[2 * v] = a;
            out[2 * v + 1] = bq;
        }
    }
}

// Clears n 64-bit words (a kernel, not a memset node: a caller may record the launch into a graph).
__global__ __launch_bounds__(SHMK_WG) void shmk_clear_words(unsigned long long *p, size_t n)
{
    for (size_t i = static_cast<size_t>(blockIdx.x) * SHMK_WG + threadIdx.x; i < n; i += static_cast<size_t>(gridDim.x) * SHMK_WG) p[i] = 0;
}

// ---- configuration 4: atomic storm -----------------------------------------------------------
template <int KIND>
__device__ __forceinline__ int64_t shmk_storm_op(const shm_dev_ctx &c, uint64_t off, int pe)
{
    if (KIND == 0) return shm_atomic_fetch_add(c, off, 1, pe);
    if (KIND == 1) {
        shm_atomic_add(c, off, 1, pe);
        return 0;
    }
    if (KIND == 2) {   // increment built from compare-swap; every failed attempt means another thread succeeded
        int64_t cur = shm_atomic_fetch(c, off, pe);
        for (;;) {
            const int64_t found = shm_atomic_compare_swap(c, off, cur, cur + 1, pe);
            if (found == cur) return cur;
            cur = found;
        }
    }
    *reinterpret_cast<volatile int64_t *>(shm_ptr(c, off, pe)) = 1;   // plain store: timing ceiling only
    return 0;
}

template <int KIND>
__global__ __launch_bounds__(SHMK_WG) void shmk_amo_storm(shm_dev_ctx c, uint64_t ctr_off, uint32_t n_ctr,
                                                          const uint16_t *__restrict__ targets, uint64_t n_items, int ops,
                                                          int64_t *__restrict__ fetched, uint64_t *__restrict__ checksum)
{
    __shared__ unsigned long long wg_sum;
    if (threadIdx.x == 0) wg_sum = 0;
    __syncthreads();
    const uint64_t g = static_cast<uint64_t>(blockIdx.x) * SHMK_WG + threadIdx.x;
    uint64_t sum = 0;
    if (g < n_items) {
        const uint16_t *t = targets + g * ops;
        int64_t *f = fetched ? fetched + g * ops : nullptr;
        int j = 0;
        if ((ops & 7) == 0) {
            for (; j < ops; j += 8) {
                const shm_u32x4 tv = *reinterpret_cast<const shm_u32x4 *>(t + j);
                const uint32_t tw[4] = {tv.x, tv.y, tv.z, tv.w};
                int64_t old[8];
#pragma unroll
                for (int q = 0; q < 8; ++q) {
                    const uint32_t tt = (q & 1) ? (tw[q >> 1] >> 16) : (tw[q >> 1] & 0xffffu);
                    old[q] = shmk_storm_op<KIND>(c, ctr_off + 8ull * (tt % n_ctr), static_cast<int>(tt / n_ctr));
                }
#pragma unroll
                for (int q = 0; q < 8; ++q) {
                    if (f) f[j + q] = old[q];
                    sum += static_cast<uint64_t>(old[q]);
                }
            }
        }
        for (; j < ops; ++j) {
            const uint32_t tt = t[j];
            const int64_t old = shmk_storm_op<KIND>(c, ctr_off + 8ull * (tt % n_ctr), static_cast<int>(tt / n_ctr));
            if (f) f[j] = old;
            sum += static_cast<uint64_t>(old);
        }
    }
    if (checksum != nullptr) {
        atomicAdd(&wg_sum, static_cast<unsigned long long>(sum));
        __syncthreads();
        if (threadIdx.x == 0) checksum[blockIdx.x] = wg_sum;
    }
}

// The same storm with the fetch-adds batched by work-groups of SHMK_STORM_WG threads.  Group b takes
// the items [b * items_per_group, (b + 1) * items_per_group) -- a multiple of SHMK_STORM_WG, so
// that the checksums stay one per SHMK_WG items -- in rounds of one item per thread, and flushes its
// counts once.
constexpr int SHMK_STORM_WG = 1024;
constexpr size_t SHMK_STORM_TABLE_BYTES = 128 * 1024;      // 16384 counters of 8 bytes, out of 160 KiB of LDS
__global__ __launch_bounds__(SHMK_STORM_WG) void shmk_amo_storm_wg(shm_dev_ctx c, uint64_t ctr_off, uint32_t n_ctr,
                                                                   const uint16_t *__restrict__ targets, uint64_t n_items, int ops,
                                                                   int64_t *__restrict__ fetched, uint64_t *__restrict__ checksum,
                                                                   uint64_t items_per_group)
{
    extern __shared__ unsigned long long shmk_storm_table[];
    __shared__ unsigned long long part_sum[SHMK_STORM_WG / SHMK_WG];
    const uint64_t first = blockIdx.x * items_per_group, last = min(n_items, first + items_per_group);
    const unsigned part = threadIdx.x / SHMK_WG;
    // Walks the group's items, calling visit(id) for every target of this thread's items.  With
    // FETCHING the values that visit returns are stored and summed.  The round loop is uniform over
    // the group (it holds barriers).
    auto walk = [&](auto visit, auto fetching) {
        constexpr bool FETCHING = decltype(fetching)::value;
        for (uint64_t r = first; r < last; r += SHMK_STORM_WG) {
            const uint64_t g = r + threadIdx.x;
            uint64_t sum = 0;
            if (g < last) {
                const uint16_t *t = targets + g * ops;
                int64_t *f = FETCHING && fetched ? fetched + g * ops : nullptr;
                int j = 0;
                if ((ops & 7) == 0) {                  // rows of whole 16-byte vectors (the table is 16-byte aligned)
                    // up to eight vectors (64 targets) are loaded before the first of them is used:
                    // one memory latency per 64 operations instead of one per eight
                    for (; j < ops; j += 64) {
                        const int nvec = min(8, (ops - j) >> 3);
                        shm_u32x4 tv[8];
#pragma unroll
                        for (int v = 0; v < 8; ++v)
                            if (v < nvec) tv[v] = *reinterpret_cast<const shm_u32x4 *>(t + j + 8 * v);
#pragma unroll
                        for (int v = 0; v < 8; ++v) {
                            if (v < nvec) {
                                const uint32_t tw[4] = {tv[v].x, tv[v].y, tv[v].z, tv[v].w};
                                int64_t old[8];
#pragma unroll
                                for (int q = 0; q < 8; ++q) old[q] = visit((q & 1) ? (tw[q >> 1] >> 16) : (tw[q >> 1] & 0xffffu));
                                if (FETCHING) {
#pragma unroll
                                    for (int q = 0; q < 8; ++q) {
                                        if (f) f[j + 8 * v + q] = old[q];
                                        sum += static_cast<uint64_t>(old[q]);
                                    }
                                }
                            }
                        }
                    }
                }
                for (; j < ops; ++j) {
                    const int64_t old = visit(t[j]);
                    if (FETCHING) {
                        if (f) f[j] = old;
                        sum += static_cast<uint64_t>(old);
                    }
                }
            }
            if (FETCHING && checksum != nullptr) {
                if (threadIdx.x < SHMK_STORM_WG / SHMK_WG) part_sum[threadIdx.x] = 0;
                __syncthreads();
                atomicAdd(&part_sum[part], static_cast<unsigned long long>(sum));
                __syncthreads();
                if (threadIdx.x % SHMK_WG == 0 && g < last) checksum[g / SHMK_WG] = part_sum[part];
                __syncthreads();
            }
        }
    };
    shmx_atomic_fetch_inc_batch_wg(
        c, ctr_off, n_ctr, shmk_storm_table,
        [&](auto count) {
            walk([&](uint32_t id) -> int64_t { count(id); return 0; }, std::false_type{});
        },
        [&](auto fetch) { walk(fetch, std::true_type{}); });
}

// The push of a long 16-byte-aligned block by ticket (fcollect: every PE's block; broadcast: the root's): the
// gridDim.x groups draw quarter-tile pieces (16 KiB: two columns per wave in each of the tile's two 32 KiB rows) of
// the block in address order, as the long put draws its pieces, and store every column to the PEs in turn, both rows
// per destination, starting with the right-hand neighbour of `p`; group 0 first moves what is left after the whole tiles,
// and the last group through sets the counter pair back.  s = the block, d0 = its offset in every destination,
// nvec = its length in vectors.  NPES > 0 fixes the number of PEs at compile time.
template <int NPES>
__device__ __forceinline__ void shmk_push_pieces_ticketed(const shm_dev_ctx &c, const shm_u32x4 *s, uint64_t d0, int p, size_t nvec,
                                                          unsigned long long *pair)
{
    __shared__ unsigned long long slots[2];
    const int npes = NPES ? NPES : c.npes;
    // The walk starts where the destinations (the same offset in equally spaced partitions) reach a
    // multiple of SHMK_STORE_LINE bytes; the vectors before it are pushed by the last group's first lanes
    // (8 PEs x 48 MiB, destination 16 / 64 / 256 bytes past a boundary: 53 / 76 / 75 % of the HBM roofline
    // walking from there, 80 % from a boundary).
    {
        size_t headv = ((SHMK_STORE_LINE - (reinterpret_cast<uintptr_t>(shm_ptr(c, d0, 0)) & (SHMK_STORE_LINE - 1))) & (SHMK_STORE_LINE - 1)) >> 4;
        if (headv > nvec) headv = nvec;
        if (blockIdx.x == gridDim.x - 1 && threadIdx.x < headv) {
            const shm_u32x4 r = shm_ld16(s + threadIdx.x);
            for (int q = 0; q < npes; ++q) shm_st16(reinterpret_cast<shm_u32x4 *>(shm_ptr(c, d0, q)) + threadIdx.x, r);
        }
        s += headv, d0 += 16 * headv, nvec -= headv;
    }
    constexpr int NQ = NPES ? NPES : 1;
    shm_u32x4 *dq[NQ];
    if (NPES) {
#pragma unroll
        for (int j = 0; j < NQ; ++j) dq[j] = reinterpret_cast<shm_u32x4 *>(shm_ptr(c, d0, (p + 1 + j) % NQ));
    }
    constexpr size_t rowv = 2048, tilev = 2 * rowv;
    constexpr unsigned PIECES = 4, CPP = 8 / PIECES;
    const unsigned wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const size_t nwhole = nvec / tilev, npieces = nwhole * PIECES;
    auto push2 = [&](size_t i, const shm_u32x4 &r0, const shm_u32x4 &r1) {
        if (NPES) {
#pragma unroll
            for (int j = 0; j < NQ; ++j) {
                shm_st16(dq[j] + i, r0);
                shm_st16(dq[j] + i + rowv, r1);
            }
        } else {
            for (int j = 0; j < npes; ++j) {
                int q = p + 1 + j;
                if (q >= npes) q -= npes;
                shm_u32x4 *d = reinterpret_cast<shm_u32x4 *>(shm_ptr(c, d0, q));
                shm_st16(d + i, r0);
                shm_st16(d + i + rowv, r1);
            }
        }
    };
    auto push = [&](size_t i, const shm_u32x4 &r) {
        for (int j = 0; j < npes; ++j) {
            int q = p + 1 + j;
            if (q >= npes) q -= npes;
            shm_st16(reinterpret_cast<shm_u32x4 *>(shm_ptr(c, d0, q)) + i, r);
        }
    };
    if (blockIdx.x == 0)                      // what is left after the whole tiles: first, while the others have all their pieces before them
        for (size_t i = nwhole * tilev + threadIdx.x; i < nvec; i += SHMK_WG) push(i, shm_ld16(s + i));
    shm_ticket_draw tk{pair, slots, gridDim.x};
    for (size_t t = blockIdx.x; t < npieces; t = tk.next()) {
        tk.ahead();
        const size_t base = (t / PIECES) * tilev + (t % PIECES) * (CPP * 64) + static_cast<size_t>(wave * 8) * 64 + lane;
#pragma unroll
        for (unsigned cc = 0; cc < CPP; ++cc) {
            const size_t i = base + cc * 64;
            const shm_u32x4 r0 = shm_ld16(s + i), r1 = shm_ld16(s + i + rowv);
            push2(i, r0, r1);
        }
    }
    if (threadIdx.x == 0) shm_tickets_done(pair, gridDim.x);
}

// ---- configuration 5a: fcollect, push --------------------------------------------------------
// PE p = blockIdx.y reads its block once and stores every vector to all PEs (inner loop over
// destinations, outer loop over addresses), starting with its right-hand neighbour.  The block is
// dealt to the PE's groups like a put.
// NPES > 0 fixes the number of PEs at compile time, so that the destination loop unrolls and the
// base-pointer lookups leave the tile loop; NPES == 0 is the general form.
// The push of one PE's block: bytes_per_pe bytes at src_off of PE p go to d0 of every PE; src_off, d0
// and bytes_per_pe are multiples of 16; the calling groups are those of blockIdx.y = p.
template <int U, int NPES>
__device__ __forceinline__ void shmk_push_block(const shm_dev_ctx &c, uint64_t d0, uint64_t src_off, size_t bytes_per_pe, int p,
                                                uint64_t ticket_pair_off)
{
    // Group-owned tiles of U rows x 32 KiB, as in shm_copy_tiles: per column U loads, then those
    // U vectors to every destination, then the next column.
    const int npes = NPES ? NPES : c.npes;
    // long blocks: the tiles start where the destinations reach a multiple of SHMK_STORE_LINE bytes, as the
    // pieces by ticket do; the vectors before it are pushed by the last group's first lanes
    if (bytes_per_pe >= SHM_LINE_HEAD_MIN_BYTES) {
        const size_t headv = ((SHMK_STORE_LINE - (reinterpret_cast<uintptr_t>(shm_ptr(c, d0, 0)) & (SHMK_STORE_LINE - 1))) & (SHMK_STORE_LINE - 1)) >> 4;
        if (blockIdx.x == gridDim.x - 1 && threadIdx.x < headv) {
            const shm_u32x4 r = shm_ld16(reinterpret_cast<const shm_u32x4 *>(shm_ptr(c, src_off, p)) + threadIdx.x);
            for (int q = 0; q < npes; ++q) shm_st16(reinterpret_cast<shm_u32x4 *>(shm_ptr(c, d0, q)) + threadIdx.x, r);
        }
        d0 += 16 * headv, src_off += 16 * headv, bytes_per_pe -= 16 * headv;
    }
    const shm_u32x4 *s = reinterpret_cast<const shm_u32x4 *>(shm_ptr(c, src_off, p));
    constexpr int NQ = NPES ? NPES : 1;
    shm_u32x4 *dq[NQ];
    if (NPES) {
#pragma unroll
        for (int j = 0; j < NQ; ++j) dq[j] = reinterpret_cast<shm_u32x4 *>(shm_ptr(c, d0, (p + 1 + j) % NQ));
    }
    const size_t nvec = bytes_per_pe >> 4;
    constexpr size_t rowv = 2048, tilev = rowv * U;
    const size_t ntiles = (nvec + tilev - 1) / tilev;
    const unsigned wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    // Which share this group takes is rotated by the PE number: the group that takes PE p's first
    // share is number p (mod groups per PE), so that the first shares of the PEs -- all there is
    // to do in a short block -- sit on different XCDs instead of all on the first one.
    const unsigned first = (blockIdx.x + gridDim.x - static_cast<unsigned>(p) % gridDim.x) % gridDim.x;
    if (ticket_pair_off) {
        shmk_push_pieces_ticketed<NPES>(c, s, d0, p, nvec, reinterpret_cast<unsigned long long *>(shm_ptr(c, ticket_pair_off, p)));
        return;
    }
    if (ntiles < gridDim.x) {
        // Short block, fewer tiles than groups: deal rows of one vector per thread instead, so that
        // as many groups as there are rows take part.
        for (size_t i = static_cast<size_t>(first) * SHMK_WG + threadIdx.x; i < nvec; i += static_cast<size_t>(gridDim.x) * SHMK_WG) {
            const shm_u32x4 r = shm_ld16(s + i);
            if (NPES) {
#pragma unroll
                for (int j = 0; j < NQ; ++j) shm_st16(dq[j] + i, r);
            } else {
                for (int j = 0; j < npes; ++j) {
                    int q = p + 1 + j;
                    if (q >= npes) q -= npes;
                    shm_st16(reinterpret_cast<shm_u32x4 *>(shm_ptr(c, d0, q)) + i, r);
                }
            }
        }
        return;
    }
    for (size_t t = first; t < ntiles; t += gridDim.x) {
        if ((t + 1) * tilev <= nvec) {            // whole tile: no predicates anywhere in the hot loop
#pragma unroll
            for (unsigned cc = 0; cc < 8; ++cc) {
                const size_t i = t * tilev + static_cast<size_t>(wave * 8 + cc) * 64 + lane;
                shm_u32x4 r[U];
#pragma unroll
                for (int u = 0; u < U; ++u) r[u] = shm_ld16(s + i + u * rowv);
                if (NPES) {
#pragma unroll
                    for (int j = 0; j < NQ; ++j)
#pragma unroll
                        for (int u = 0; u < U; ++u) shm_st16(dq[j] + i + u * rowv, r[u]);
                } else {
                    for (int j = 0; j < npes; ++j) {
                        int q = p + 1 + j;
                        if (q >= npes) q -= npes;
                        shm_u32x4 *d = reinterpret_cast<shm_u32x4 *>(shm_ptr(c, d0, q));
#pragma unroll
                        for (int u = 0; u < U; ++u) shm_st16(d + i + u * rowv, r[u]);
                    }
                }
            }
        } else {                                  // the last, partial tile
            for (unsigned cc = 0; cc < 8; ++cc) {
                for (int u = 0; u < U; ++u) {
                    const size_t i = t * tilev + static_cast<size_t>(wave * 8 + cc) * 64 + lane + u * rowv;
                    if (i >= nvec) continue;
                    const shm_u32x4 r = shm_ld16(s + i);
                    for (int j = 0; j < npes; ++j) {
                        int q = p + 1 + j;
                        if (q >= npes) q -= npes;
                        shm_st16(reinterpret_cast<shm_u32x4 *>(shm_ptr(c, d0, q)) + i, r);
                    }
                }
            }
        }
    }
}

template <int U, int NPES>
__global__ __launch_bounds__(SHMK_WG) void shmk_fcollect_vec(shm_dev_ctx c, uint64_t dst_off, uint64_t src_off, size_t bytes_per_pe,
                                                             uint64_t ticket_pair_off)
{
    const int p = blockIdx.y;
    shmk_push_block<U, NPES>(c, dst_off + static_cast<uint64_t>(p) * bytes_per_pe, src_off, bytes_per_pe, p, ticket_pair_off);
}

// Any alignment or length: PE p's block is pushed to every PE like a broadcast rooted at p -- each
// vector loaded once and stored to all PEs where source and destination are 16-byte aligned, one
// multi-group put per destination otherwise.
__global__ __launch_bounds__(SHMK_WG) void shmk_fcollect_any(shm_dev_ctx c, uint64_t dst_off, uint64_t src_off, size_t bytes_per_pe)
{
    const int p = blockIdx.y;
    shmx_broadcast_push(c, p, dst_off + static_cast<uint64_t>(p) * bytes_per_pe, src_off, bytes_per_pe, blockIdx.x, gridDim.x);
}

// collect: as fcollect with a block size per PE; the launcher passes every PE's size and the offset
// of its block in the destination (exclusive prefix sum of the sizes).
struct shmk_collect_table {
    uint64_t at[SHM_MAX_PES];        // destination offset of PE p's block, relative to dst_off
    uint64_t nbytes[SHM_MAX_PES];
};

// A block whose place in the destination and whose length are multiples of 16 bytes is pushed like
// fcollect's (tiles, or pieces by ticket when the launcher passes the counters); any other block the
// general way.
template <int NPES>
__global__ __launch_bounds__(SHMK_WG) void shmk_collect(shm_dev_ctx c, uint64_t dst_off, uint64_t src_off, shmk_collect_table t,
                                                        uint64_t ticket_pair_off)
{
    const int p = blockIdx.y;
    const uint64_t d0 = dst_off + t.at[p];
    if (((d0 | src_off | t.nbytes[p]) & 15) == 0)
        shmk_push_block<2, NPES>(c, d0, src_off, t.nbytes[p], p, ticket_pair_off);
    else
        shmx_broadcast_push(c, p, d0, src_off, t.nbytes[p], blockIdx.x, gridDim.x);
}

// Team grids (n_wg, npes) whose npes groups with the same blockIdx.x read the SAME source bytes
// (the duplicate reduction): groups go to the 8 XCDs round-robin in linear order and each XCD has
// its own L2, so the npes readers of one share are renumbered to be consecutive groups of one XCD
// -- they run together and all but the first find the source in that L2 instead of in HBM.
// Needs gridDim.x to be a multiple of 8; otherwise the plain numbering stays.
__device__ __forceinline__ void shmk_duplicate_coords(int npes, unsigned &part, int &q)
{
    part = blockIdx.x;
    q = blockIdx.y;
    if ((gridDim.x & 7u) == 0) {
        const unsigned lin = blockIdx.x + gridDim.x * blockIdx.y;
        const unsigned xcd = lin & 7u, j = lin >> 3;
        q = static_cast<int>(j % npes);
        part = (j / npes) * 8 + xcd;
    }
}

// Vectors per PE of a split reduction over nvec 16-byte vectors: an equal share, and from
// SHMK_OWNED_MIN_TILES tiles on a whole number of 64 KiB tiles, so that every PE's slice starts on
// a tile boundary whatever the number of PEs (the last PEs then take what is left; with slices that
// began at any 16 bytes 6 PEs x 128 MiB measured 57 % of the HBM roofline).
// Vectors before the first slice of a split reduction: the slices start where the destinations (the
// same offset in equally spaced partitions) reach a multiple of SHMK_STORE_LINE bytes, and PE 0's last
// group folds the vectors before that place (8 PEs x 64 MiB, destination 16 bytes past a boundary:
// 56.8 % of the HBM roofline with slices from the destination's first byte).
__device__ __forceinline__ size_t shmk_split_head(const shm_dev_ctx &c, uint64_t dst_off, size_t nvec)
{
    const size_t headv = ((SHMK_STORE_LINE - (reinterpret_cast<uintptr_t>(shm_ptr(c, dst_off, 0)) & (SHMK_STORE_LINE - 1))) & (SHMK_STORE_LINE - 1)) >> 4;
    return headv < nvec ? headv : nvec;
}

__host__ __device__ inline size_t shmk_split_share(size_t nvec, int npes)
{
    const size_t share = (nvec + npes - 1) / npes;
    return share < size_t(4096) * SHMK_OWNED_MIN_TILES ? share : (share + 4095) / 4096 * 4096;
}

// ---- configuration 5b: float32 sum-reduce ---------------------------------------------------
// Element i of the result is ((x0[i] + x1[i]) + x2[i]) + ... in PE order, on every PE.
// SPLIT = false: PE q = blockIdx.y computes all elements and stores to its own destination.
// SPLIT = true : PE q computes the q-th share of the vectors and stores it to every PE.
template <bool SPLIT>
__global__ __launch_bounds__(SHMK_WG) void shmk_reduce_sum_f32_vec(shm_dev_ctx c, uint64_t dst_off, uint64_t src_off, size_t nvec,
                                                                   uint64_t ticket_pair_off)
{
    constexpr int U = 2;
    const int npes = c.npes;
    int q = blockIdx.y;
    unsigned part = blockIdx.x;
    if (!SPLIT) shmk_duplicate_coords(npes, part, q);
    size_t first = 0, count = nvec, headv = 0;
    if (SPLIT) {
        headv = shmk_split_head(c, dst_off, nvec);
        const size_t share = shmk_split_share(nvec - headv, npes);
        first = min(nvec, headv + q * share);
        count = min(nvec, first + share) - first;
    }
    const uint64_t so = src_off + 16 * first, dof = dst_off + 16 * first;
    const shm_deal k = shm_deal_make<U>(count, part, gridDim.x, threadIdx.x, SHMK_WG);
    // duplicate: the other PEs' groups on this XCD read the same vectors, so they are kept in L2
    auto load = [&](const shm_f32x4 *a) { return SPLIT ? __builtin_nontemporal_load(a) : *a; };
    auto emit = [&](size_t i, shm_f32x4 r) {
        if (SPLIT) {
            for (int t = 0; t < npes; ++t) {
                int w = q + t;                      // own copy first, then the others in ring order
                if (w >= npes) w -= npes;
                __builtin_nontemporal_store(r, reinterpret_cast<shm_f32x4 *>(shm_ptr(c, dof, w)) + i);
            }
        } else {
            __builtin_nontemporal_store(r, reinterpret_cast<shm_f32x4 *>(shm_ptr(c, dof, q)) + i);
        }
    };
    // whole tiles: U vectors per thread, rowv apart, starting at vector i
    auto tile_part = [&](size_t i, size_t rowv) {
        shm_f32x4 r[U];
#pragma unroll
        for (int u = 0; u < U; ++u)
            r[u] = load(reinterpret_cast<const shm_f32x4 *>(shm_ptr(c, so, 0)) + i + u * rowv);
        // The other PEs' vectors four PEs at a time (then two, then one): the loads of a batch are
        // all issued before the first add waits for one, the adds stay in PE order.
        int p = 1;
        for (; p + 3 < npes; p += 4) {
            shm_f32x4 v[4][U];
#pragma unroll
            for (int j = 0; j < 4; ++j)
#pragma unroll
                for (int u = 0; u < U; ++u) v[j][u] = load(reinterpret_cast<const shm_f32x4 *>(shm_ptr(c, so, p + j)) + i + u * rowv);
#pragma unroll
            for (int j = 0; j < 4; ++j)
#pragma unroll
                for (int u = 0; u < U; ++u) r[u].x += v[j][u].x, r[u].y += v[j][u].y, r[u].z += v[j][u].z, r[u].w += v[j][u].w;
        }
        for (; p + 1 < npes; p += 2) {
            shm_f32x4 v[2][U];
#pragma unroll
            for (int j = 0; j < 2; ++j)
#pragma unroll
                for (int u = 0; u < U; ++u) v[j][u] = load(reinterpret_cast<const shm_f32x4 *>(shm_ptr(c, so, p + j)) + i + u * rowv);
#pragma unroll
            for (int j = 0; j < 2; ++j)
#pragma unroll
                for (int u = 0; u < U; ++u) r[u].x += v[j][u].x, r[u].y += v[j][u].y, r[u].z += v[j][u].z, r[u].w += v[j][u].w;
        }
        for (; p < npes; ++p) {
            const shm_f32x4 *sp = reinterpret_cast<const shm_f32x4 *>(shm_ptr(c, so, p));
            shm_f32x4 v[U];
#pragma unroll
            for (int u = 0; u < U; ++u) v[u] = load(sp + i + u * rowv);
#pragma unroll
            for (int u = 0; u < U; ++u) r[u].x += v[u].x, r[u].y += v[u].y, r[u].z += v[u].z, r[u].w += v[u].w;
        }
        if (SPLIT) {
            // destination by destination, both rows each (own copy first, then the others in ring
            // order): 75.4 % of the HBM roofline at 8 PEs x 64 MiB against 71.8 % row by row
            for (int t = 0; t < npes; ++t) {
                int w = q + t;
                if (w >= npes) w -= npes;
                shm_f32x4 *dw = reinterpret_cast<shm_f32x4 *>(shm_ptr(c, dof, w));
#pragma unroll
                for (int u = 0; u < U; ++u) __builtin_nontemporal_store(r[u], dw + i + u * rowv);
            }
            return;
        }
#pragma unroll
        for (int u = 0; u < U; ++u) emit(i + u * rowv, r[u]);
    };
    // Split: with enough tiles to fill the chip a PE's slice is walked on group-owned tiles of two
    // 32 KiB rows (wave w takes columns 8w .. 8w+7; groups beyond the number of tiles have nothing to
    // do), measured 3-4 points of the HBM roofline better than tiles shared by eight groups; what is
    // left after the whole tiles is dealt one vector per lane over all groups either way.
    constexpr size_t own_rowv = 2048, own_tilev = U * own_rowv;
    const bool owned = SPLIT && count / own_tilev >= SHMK_OWNED_MIN_TILES;
    size_t rem_lane = k.rem_lane;
    if (owned && ticket_pair_off) {
        // by ticket: the PE's groups (the launcher runs one per compute unit in all) draw quarter
        // tiles of the slice in address order from the pair in PE q's tail
        __shared__ unsigned long long slots[2];
        constexpr unsigned PIECES = SHMK_REDUCE_PIECES, CPP = 8 / PIECES;
        const size_t ntiles = count / own_tilev, npieces = ntiles * PIECES;
        const unsigned wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
        unsigned long long *pair = reinterpret_cast<unsigned long long *>(shm_ptr(c, ticket_pair_off, q));
        shm_ticket_draw tk{pair, slots, gridDim.x};
        for (size_t t = part; t < npieces; t = tk.next()) {
            tk.ahead();
            const size_t base = (t / PIECES) * own_tilev + (t % PIECES) * (CPP * 64) + static_cast<size_t>(wave * 8) * 64 + lane;
#pragma unroll
            for (unsigned cc = 0; cc < CPP; ++cc) tile_part(base + cc * 64, own_rowv);
        }
        if (threadIdx.x == 0) shm_tickets_done(pair, gridDim.x);
        rem_lane = ntiles * own_tilev + static_cast<size_t>(part) * SHMK_WG + threadIdx.x;
    } else if (owned) {
        const size_t ntiles = count / own_tilev;
        const unsigned wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
        for (size_t t = part; t < ntiles; t += gridDim.x) {
#pragma unroll 2
            for (unsigned cc = 0; cc < 8; ++cc) tile_part(t * own_tilev + static_cast<size_t>(wave * 8 + cc) * 64 + lane, own_rowv);
        }
        rem_lane = ntiles * own_tilev + static_cast<size_t>(part) * SHMK_WG + threadIdx.x;
    } else {
        for (size_t t = k.vb; t < k.ntiles; t += k.nvb) tile_part(t * k.tilev + k.col, k.rowv);
    }
    for (size_t i = rem_lane; i < count; i += k.rem_step) {
        shm_f32x4 r = load(reinterpret_cast<const shm_f32x4 *>(shm_ptr(c, so, 0)) + i);
        for (int p = 1; p < npes; ++p) {
            const shm_f32x4 v = load(reinterpret_cast<const shm_f32x4 *>(shm_ptr(c, so, p)) + i);
            r.x += v.x, r.y += v.y, r.z += v.z, r.w += v.w;
        }
        emit(i, r);
    }
    if (SPLIT && q == 0 && part == gridDim.x - 1 && threadIdx.x < headv) {       // the vectors before the first slice
        shm_f32x4 r = load(reinterpret_cast<const shm_f32x4 *>(shm_ptr(c, src_off, 0)) + threadIdx.x);
        for (int p = 1; p < npes; ++p) {
            const shm_f32x4 v = load(reinterpret_cast<const shm_f32x4 *>(shm_ptr(c, src_off, p)) + threadIdx.x);
            r.x += v.x, r.y += v.y, r.z += v.z, r.w += v.w;
        }
        for (int w = 0; w < npes; ++w) __builtin_nontemporal_store(r, reinterpret_cast<shm_f32x4 *>(shm_ptr(c, dst_off, w)) + threadIdx.x);
    }
}

// Scalar form for the last nelems % 4 elements and for offsets that are not 16-byte aligned:
// elements [first, nelems), every PE q = blockIdx.y writes its own destination.
__global__ __launch_bounds__(SHMK_WG) void shmk_reduce_sum_f32_scalar(shm_dev_ctx c, uint64_t dst_off, uint64_t src_off, size_t first,
                                                                      size_t nelems)
{
    const int q = blockIdx.y, npes = c.npes;
    const size_t stride = static_cast<size_t>(gridDim.x) * SHMK_WG;
    for (size_t i = first + static_cast<size_t>(blockIdx.x) * SHMK_WG + threadIdx.x; i < nelems; i += stride) {
        float r = reinterpret_cast<const float *>(shm_ptr(c, src_off, 0))[i];
        for (int p = 1; p < npes; ++p) r += reinterpret_cast<const float *>(shm_ptr(c, src_off, p))[i];
        reinterpret_cast<float *>(shm_ptr(c, dst_off, q))[i] = r;
    }
}

// ---- device-side synchronisation among PEs ------------------------------------------------------
// One group per PE (blockIdx.x = PE).  Round r: PE p puts its block into slot p of PE (p+1+r) mod
// npes, all PEs meet in a device barrier, then p copies the slot that was just filled for it (the
// block of PE (p-1-r) mod npes) to acc_off + r*n.  Without a working barrier the copy reads stale
// bytes.
__global__ __launch_bounds__(SHMK_WG) void shmk_barrier_exchange(shm_dev_ctx c, uint64_t dst_off, uint64_t src_off, uint64_t acc_off,
                                                                 size_t n, int rounds)
{
    const int me = blockIdx.x, npes = c.npes;
    for (int r = 0; r < rounds; ++r) {
        const int to = (me + 1 + r) % npes;
        int from = (me - 1 - r) % npes;
        if (from < 0) from += npes;
        shmx_putmem_wg(c, me, dst_off + static_cast<uint64_t>(me) * n, src_off, n, to);
        shmx_barrier_all_wg(c, me);
        shmx_getmem_wg(c, me, acc_off + static_cast<uint64_t>(r) * n, dst_off + static_cast<uint64_t>(from) * n, n, me);
    }
}

// `rounds` syncs by one group per PE; device clock around them.
__global__ __launch_bounds__(SHMK_WG) void shmk_sync_all(shm_dev_ctx c, int rounds, int with_quiet, unsigned long long *ticks)
{
    const int me = blockIdx.x;
    const unsigned long long t0 = wall_clock64();
    for (int r = 0; r < rounds; ++r) {
        if (with_quiet)
            shmx_barrier_all_wg(c, me);
        else
            shmx_sync_all_wg(c, me);
    }
    const unsigned long long t1 = wall_clock64();
    if (threadIdx.x == 0) {
        atomicMin(&ticks[0], t0);
        atomicMax(&ticks[1], t1);
    }
}

// ticket_pair_off != 0 (long blocks; offsets 16-byte aligned): the groups draw pieces by ticket from the root's pair.
__global__ __launch_bounds__(SHMK_WG) void shmk_broadcast(shm_dev_ctx c, uint64_t dst_off, uint64_t src_off, size_t n, int root,
                                                          uint64_t ticket_pair_off)
{
    if (ticket_pair_off == 0) {
        shmx_broadcast_push(c, root, dst_off, src_off, n, blockIdx.x, gridDim.x);
        return;
    }
    const char *src = shm_ptr(c, src_off, root);
    shmk_push_pieces_ticketed<0>(c, reinterpret_cast<const shm_u32x4 *>(src), dst_off, root, n >> 4,
                                 reinterpret_cast<unsigned long long *>(shm_ptr(c, ticket_pair_off, root)));
    if (blockIdx.x == 0)
        for (size_t b = (n & ~static_cast<size_t>(15)) + threadIdx.x; b < n; b += SHMK_WG) {       // the last n mod 16 bytes
            const char v = src[b];
            for (int q = 0; q < c.npes; ++q) shm_ptr(c, dst_off, q)[b] = v;
        }
}

// ---- the reduction matrix (paper section "Collective Operations", reduction paragraph) ------------
// min, max, sum, product, and, or, xor over 8..64-bit integers; min, max, sum, product over float
// and double.  Work is split by address across threads; every thread loads one 16-byte vector from
// each PE in PE order 0..npes-1, folds them element by element and stores the result to its own
// PE's destination; every PE (blockIdx.y) duplicates the computation, so no PE waits for another.
// Integer sums and products wrap (computed in the unsigned type); min/max keep the earlier operand
// on ties, which also fixes the sign of a zero.
template <typename T, int OP, bool SPLIT>
__global__ __launch_bounds__(SHMK_WG) void shmk_reduce(shm_dev_ctx c, uint64_t dst_off, uint64_t src_off, size_t nelems,
                                                       uint64_t ticket_pair_off)
{
    // SPLIT false: every PE folds the whole vector into its own destination (the paper's method: no
    // PE waits for another).  SPLIT true: the method the paper names for very large reductions --
    // the vector is divided by address across PEs; PE q folds only its slice and pushes the result
    // to every PE's destination, so each source byte is read once instead of npes times.  A kernel
    // per method: with the method as a run-time argument every load carried the choice between its
    // two forms, and the split reduction of 8 x 64 MiB measured 70.9 % of the HBM roofline against 72.1 %.
    constexpr bool split = SPLIT;
    constexpr int EPV = 16 / sizeof(T);
    union vec {
        shm_u32x4 v;
        T e[EPV];
    };
    const int npes = c.npes;
    int q = blockIdx.y;
    unsigned part = blockIdx.x;
    if (!split) shmk_duplicate_coords(npes, part, q);
    const int d0 = split ? 0 : q, d1 = split ? npes : q + 1;
    const size_t nvec = nelems / EPV;
    size_t vlo = 0, vhi = nvec, headv = 0;
    if (split) {
        headv = shmk_split_head(c, dst_off, nvec);
        const size_t per_pe = shmk_split_share(nvec - headv, npes);
        vlo = min(nvec, headv + q * per_pe);
        vhi = min(nvec, vlo + per_pe);
    }
    const size_t per = (vhi - vlo + gridDim.x - 1) / gridDim.x;
    const size_t lo = min(vhi, vlo + part * per), hi = min(vhi, lo + per);
    // duplicate: the other PEs' groups on this XCD read the same vectors, so they are kept in L2
    auto load = [&](const shm_u32x4 *a) { return split ? shm_ld16(a) : *a; };
    // two vectors per thread and pass (the second one a group's width further on), so that twice as
    // many loads are in flight; then whatever is left, one vector per thread
    auto fold2 = [&](size_t i, size_t i2) {
        vec r0, r1;
        r0.v = load(reinterpret_cast<const shm_u32x4 *>(shm_ptr(c, src_off, 0)) + i);
        r1.v = load(reinterpret_cast<const shm_u32x4 *>(shm_ptr(c, src_off, 0)) + i2);
        // the other PEs' vectors four PEs at a time, then two, then one: a batch's loads are all
        // issued before the first fold waits for one; the folds stay in PE order
        int p = 1;
        for (; p + 3 < npes; p += 4) {
            vec x0[4], x1[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                x0[j].v = load(reinterpret_cast<const shm_u32x4 *>(shm_ptr(c, src_off, p + j)) + i);
                x1[j].v = load(reinterpret_cast<const shm_u32x4 *>(shm_ptr(c, src_off, p + j)) + i2);
            }
#pragma unroll
            for (int j = 0; j < 4; ++j) {
#pragma unroll
                for (int k = 0; k < EPV; ++k) r0.e[k] = shm_combine<T, OP>(r0.e[k], x0[j].e[k]);
#pragma unroll
                for (int k = 0; k < EPV; ++k) r1.e[k] = shm_combine<T, OP>(r1.e[k], x1[j].e[k]);
            }
        }
        for (; p + 1 < npes; p += 2) {
            vec x0[2], x1[2];
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                x0[j].v = load(reinterpret_cast<const shm_u32x4 *>(shm_ptr(c, src_off, p + j)) + i);
                x1[j].v = load(reinterpret_cast<const shm_u32x4 *>(shm_ptr(c, src_off, p + j)) + i2);
            }
#pragma unroll
            for (int j = 0; j < 2; ++j) {
#pragma unroll
                for (int k = 0; k < EPV; ++k) r0.e[k] = shm_combine<T, OP>(r0.e[k], x0[j].e[k]);
#pragma unroll
                for (int k = 0; k < EPV; ++k) r1.e[k] = shm_combine<T, OP>(r1.e[k], x1[j].e[k]);
            }
        }
        for (; p < npes; ++p) {
            vec x0, x1;
            x0.v = load(reinterpret_cast<const shm_u32x4 *>(shm_ptr(c, src_off, p)) + i);
            x1.v = load(reinterpret_cast<const shm_u32x4 *>(shm_ptr(c, src_off, p)) + i2);
#pragma unroll
            for (int k = 0; k < EPV; ++k) r0.e[k] = shm_combine<T, OP>(r0.e[k], x0.e[k]);
#pragma unroll
            for (int k = 0; k < EPV; ++k) r1.e[k] = shm_combine<T, OP>(r1.e[k], x1.e[k]);
        }
        for (int t = d0; t < d1; ++t) {           // split: own copy first, then the others in ring order
            const int d = !split ? t : q + t < npes ? q + t : q + t - npes;
            shm_st16(reinterpret_cast<shm_u32x4 *>(shm_ptr(c, dst_off, d)) + i, r0.v);
            shm_st16(reinterpret_cast<shm_u32x4 *>(shm_ptr(c, dst_off, d)) + i2, r1.v);
        }
    };
    auto fold1 = [&](size_t i) {
        vec r;
        r.v = load(reinterpret_cast<const shm_u32x4 *>(shm_ptr(c, src_off, 0)) + i);
        for (int p = 1; p < npes; ++p) {
            vec x;
            x.v = load(reinterpret_cast<const shm_u32x4 *>(shm_ptr(c, src_off, p)) + i);
#pragma unroll
            for (int k = 0; k < EPV; ++k) r.e[k] = shm_combine<T, OP>(r.e[k], x.e[k]);
        }
        for (int d = d0; d < d1; ++d) shm_st16(reinterpret_cast<shm_u32x4 *>(shm_ptr(c, dst_off, d)) + i, r.v);
    };
    // Split: a PE's slice is walked on group-owned tiles of two 32 KiB rows (the order of the long
    // put: wave w takes columns 8w .. 8w+7, two vectors 32 KiB apart per column) when there are enough
    // tiles to fill the chip -- measured 3-4 points of the HBM roofline better than contiguous slices;
    // groups beyond the number of tiles have nothing to do.  Otherwise contiguous slices per group.
    constexpr size_t rowv = 2048, tilev = 2 * rowv;
    const size_t ntiles = (vhi - vlo) / tilev;
    if (split && ntiles >= SHMK_OWNED_MIN_TILES) {
        const unsigned wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
        if (ticket_pair_off) {
            // by ticket, as in shmk_reduce_sum_f32_vec: quarter tiles of the slice in address order
            __shared__ unsigned long long slots[2];
            constexpr unsigned PIECES = SHMK_REDUCE_PIECES, CPP = 8 / PIECES;
            unsigned long long *pair = reinterpret_cast<unsigned long long *>(shm_ptr(c, ticket_pair_off, q));
            shm_ticket_draw tk{pair, slots, gridDim.x};
            for (size_t t = part; t < ntiles * PIECES; t = tk.next()) {
                tk.ahead();
                const size_t base = vlo + (t / PIECES) * tilev + (t % PIECES) * (CPP * 64) + static_cast<size_t>(wave * 8) * 64 + lane;
#pragma unroll
                for (unsigned cc = 0; cc < CPP; ++cc) fold2(base + cc * 64, base + cc * 64 + rowv);
            }
            if (threadIdx.x == 0) shm_tickets_done(pair, gridDim.x);
        } else
        for (size_t t = part; t < ntiles; t += gridDim.x) {
#pragma unroll 2
            for (unsigned cc = 0; cc < 8; ++cc) {
                const size_t i = vlo + t * tilev + static_cast<size_t>(wave * 8 + cc) * 64 + lane;
                fold2(i, i + rowv);
            }
        }
        for (size_t i = vlo + ntiles * tilev + static_cast<size_t>(part) * SHMK_WG + threadIdx.x; i < vhi;
             i += static_cast<size_t>(gridDim.x) * SHMK_WG)
            fold1(i);
    } else {
        size_t i = lo + threadIdx.x;
        for (; i + SHMK_WG < hi; i += 2 * SHMK_WG) fold2(i, i + SHMK_WG);
        for (; i < hi; i += SHMK_WG) fold1(i);
    }
    if (split && q == 0 && part == gridDim.x - 1 && threadIdx.x < headv) fold1(threadIdx.x);       // the vectors before the first slice
    // the last nelems mod EPV elements, one thread each
    const size_t t = nvec * EPV + threadIdx.x;
    if (part == 0 && (!split || q == 0) && t < nelems) {
        T r = reinterpret_cast<const T *>(shm_ptr(c, src_off, 0))[t];
        for (int p = 1; p < npes; ++p) r = shm_combine<T, OP>(r, reinterpret_cast<const T *>(shm_ptr(c, src_off, p))[t]);
        for (int d = d0; d < d1; ++d) reinterpret_cast<T *>(shm_ptr(c, dst_off, d))[t] = r;
    }
}
