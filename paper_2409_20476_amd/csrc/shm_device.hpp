// Device-side OpenSHMEM API for gfx950: the functions a kernel embeds to move data between
// logical PEs.  Header-only; every function is __device__ and inlined into its caller.
//
// Naming follows the paper's section "Proposed Device APIs": shm_* are per-thread calls, shmx_*
// are the collaborative extensions, which EVERY thread of the wave / work-group must reach with
// identical arguments.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "shm_release_algo.hpp"

#define SHM_MAX_PES 32

// Per-launch view of the context, passed to kernels by value (it lives in the kernel-argument
// segment and is read with scalar loads).  base[] plays the role of the paper's local-PE table
// plus heap-offset array (section "Inter-node and Intra-node Communication"): one lookup gives
// the target heap's base address.
// Device view of the reverse-offload ring (all null when the host proxy is not running).
struct shm_offload_dev {
    uint32_t *ring;                  // pinned host memory: SHM_OFFLOAD_SLOTS messages of 16 words
    uint32_t *completion;            // pinned host memory: completion words, written by the host
    const uint64_t *consumed;        // pinned host memory: requests the host has taken (flow control)
    unsigned long long *head;        // device memory: next request index
    unsigned long long *comp_head;   // device memory: next completion index
    unsigned long long *consumed_seen;   // device memory: the largest `consumed` any sender has read from the host
};

struct shm_dev_ctx {
    char *base[SHM_MAX_PES];
    uint64_t *status;        // host-pinned word; set to 1 when a bounded wait expired
    uint64_t wait_ticks;     // bound for every wait, in wall_clock64() ticks
    uint64_t stride;         // base[p] == base[0] + p * stride for every p (equally spaced partitions), else 0
    uint64_t internal_off;   // offset of the library's own tail of every partition
    shm_offload_dev off;
    int npes;
};

// Words in the library's tail of every partition (byte offsets from internal_off).
#define SHMD_INTERNAL_SYNC_COUNT 33024u   // uint64: increments received from the other PEs' syncs
#define SHMD_INTERNAL_SYNC_EPOCH 33032u   // uint64: syncs this PE has completed

typedef uint32_t shm_u32x4 __attribute__((ext_vector_type(4)));

enum { SHMD_SIGNAL_SET = 0, SHMD_SIGNAL_ADD = 1 };

// Memory orders of the atomics that publish a payload (the arrival counters of a message shared by
// several groups, and the signal word).  The library's build stores such payloads write-through,
// waits for their acknowledgement and then needs no ordering from the atomic itself (relaxed).
// Built with -DSHM_SIGNAL_FULL_RELEASE the same atomics are release / acquire-release operations,
// with the cache write-backs that implies: the textbook form, kept as a second library that the
// signalling tests are run against as a cross-check of the relaxed form.
#ifdef SHM_SIGNAL_FULL_RELEASE
#define SHMD_ARRIVE_ORDER __ATOMIC_ACQ_REL
#define SHMD_SIGNAL_ORDER __ATOMIC_RELEASE
#else
#define SHMD_ARRIVE_ORDER __ATOMIC_RELAXED
#define SHMD_SIGNAL_ORDER __ATOMIC_RELAXED
#endif
enum { SHMD_CMP_EQ = 0, SHMD_CMP_NE = 1, SHMD_CMP_GT = 2, SHMD_CMP_GE = 3, SHMD_CMP_LT = 4, SHMD_CMP_LE = 5 };

// Address rule of the paper's section "Remote Memory Access": same offset, target PE's base.  With
// equally spaced partitions the base is computed instead of looked up, which keeps table loads out
// of inner loops that visit every PE.
__device__ __forceinline__ char *shm_ptr(const shm_dev_ctx &c, uint64_t off, int pe)
{
    if (__builtin_expect(c.stride != 0, 1)) return c.base[0] + static_cast<uint64_t>(pe) * c.stride + off;
    return c.base[pe] + off;
}

// ------------------------------------------------------------------------------------------
// Cooperative byte copy: `nthr` threads (this one is `tid`) copy n bytes, any alignment.
// Destination-aligned 16-byte nontemporal stores; 16-byte nontemporal loads, U of them in flight
// per lane before the first store.  When source and destination disagree modulo 16 the source is
// read as aligned 16-byte words and re-aligned in registers, so no access is ever misaligned.
// ------------------------------------------------------------------------------------------
__device__ __forceinline__ shm_u32x4 shm_ld16(const shm_u32x4 *p) { return __builtin_nontemporal_load(p); }

// Store policies.  SHM_ST_STREAM: nontemporal, the fastest for bulk data that nobody waits for
// inside the kernel.  SHM_ST_THROUGH: written through the XCD's L2 (the sc1 bit, which is how an
// agent-scope atomic store is encoded), for payloads that a release follows at once: the release's
// cache write-back then finds nothing dirty and costs a fraction of a microsecond less per group,
// measured 5x cheaper when many groups release together.  Both are ordinary stores as far as the
// memory model goes; the release fence and the signal atomic that follow are unchanged.
enum { SHM_ST_STREAM = 0, SHM_ST_THROUGH = 1 };
template <int POLICY = SHM_ST_STREAM>
__device__ __forceinline__ void shm_st16(shm_u32x4 *p, shm_u32x4 v)
{
    if (POLICY == SHM_ST_THROUGH)
        // The s_nop belongs to the store: the hardware reads the upper half of a store's 16 data
        // bytes one issue cycle late, and a vector-ALU write to those registers in that window
        // corrupts them.  The compiler pads its own stores; it cannot see inside this one.
        asm volatile("global_store_dwordx4 %0, %1, off sc1\n\ts_nop 1" ::"v"(p), "v"(v) : "memory");
    else
        __builtin_nontemporal_store(v, p);
}

// bytes [8*sh .. 8*sh+32) of the 64-bit value hi:lo, sh in 0..3
__device__ __forceinline__ uint32_t shm_alignbyte(uint32_t hi, uint32_t lo, uint32_t sh)
{
    return __builtin_amdgcn_alignbyte(hi, lo, sh);
}

template <int W>   // W = whole words of shift (0..3); sh = remaining bytes (0..3)
__device__ __forceinline__ shm_u32x4 shm_realign(shm_u32x4 lo, shm_u32x4 hi, uint32_t sh)
{
    const uint32_t w[8] = {lo.x, lo.y, lo.z, lo.w, hi.x, hi.y, hi.z, hi.w};
    shm_u32x4 r;
    r.x = shm_alignbyte(w[W + 1], w[W + 0], sh);
    r.y = shm_alignbyte(w[W + 2], w[W + 1], sh);
    r.z = shm_alignbyte(w[W + 3], w[W + 2], sh);
    r.w = shm_alignbyte(w[W + 4], w[W + 3], sh);
    return r;
}

template <int U, int POLICY = SHM_ST_STREAM>
__device__ __forceinline__ void shm_copy_body_aligned(shm_u32x4 *d, const shm_u32x4 *s, size_t nvec, unsigned tid,
                                                      unsigned nthr)
{
    size_t i = tid;
    const size_t step = nthr;
    for (; i + (U - 1) * step < nvec; i += U * step) {
        shm_u32x4 r[U];
#pragma unroll
        for (int u = 0; u < U; ++u) r[u] = shm_ld16(s + i + u * step);
#pragma unroll
        for (int u = 0; u < U; ++u) shm_st16<POLICY>(d + i + u * step, r[u]);
    }
    for (; i < nvec; i += step) shm_st16<POLICY>(d + i, shm_ld16(s + i));
}

template <int W, int POLICY = SHM_ST_STREAM>
__device__ __forceinline__ void shm_copy_body_shifted(shm_u32x4 *d, const shm_u32x4 *sa, size_t nvec, uint32_t sh,
                                                      unsigned tid, unsigned nthr)
{
    // sa is the aligned word holding the first source byte; vector i needs words i and i+1.
    // Word i+1 always contains at least one byte of the source range, so it is mapped.
    for (size_t i = tid; i < nvec; i += nthr) {
        const shm_u32x4 lo = shm_ld16(sa + i);
        const shm_u32x4 hi = shm_ld16(sa + i + 1);
        shm_st16<POLICY>(d + i, shm_realign<W>(lo, hi, sh));
    }
}

template <int POLICY = SHM_ST_STREAM>
__device__ __forceinline__ void shm_st1(char *p, char v)
{
    if (POLICY == SHM_ST_THROUGH)
        asm volatile("global_store_byte %0, %1, off sc1" ::"v"(p), "v"(static_cast<int>(v)) : "memory");
    else
        *p = v;
}

template <int POLICY = SHM_ST_STREAM>
__device__ __forceinline__ void shm_st8(char *p, uint64_t v)
{
    if (POLICY == SHM_ST_THROUGH)
        asm volatile("global_store_dwordx2 %0, %1, off sc1" ::"v"(p), "v"(v) : "memory");
    else
        *reinterpret_cast<uint64_t *>(p) = v;
}
template <int POLICY = SHM_ST_STREAM>
__device__ __forceinline__ void shm_st4(char *p, uint32_t v)
{
    if (POLICY == SHM_ST_THROUGH)
        asm volatile("global_store_dword %0, %1, off sc1" ::"v"(p), "v"(v) : "memory");
    else
        *reinterpret_cast<uint32_t *>(p) = v;
}

// Fewer than 16 bytes by ONE thread: an 8- and a 4-byte piece where both addresses allow, bytes for
// the rest (a thread's byte stores follow one another at a memory round trip each: 8 bytes as bytes
// measure 2.3 us, as one piece what a 16-byte put takes).
template <int POLICY = SHM_ST_STREAM>
__device__ __forceinline__ void shm_copy_below16(char *dst, const char *src, size_t len)
{
    const uintptr_t both = reinterpret_cast<uintptr_t>(dst) | reinterpret_cast<uintptr_t>(src);
    size_t i = 0;
    if (len >= 8 && (both & 7) == 0) {
        shm_st8<POLICY>(dst, *reinterpret_cast<const uint64_t *>(src));
        i = 8;
    }
    if (len - i >= 4 && (both & 3) == 0) {
        shm_st4<POLICY>(dst + i, *reinterpret_cast<const uint32_t *>(src + i));
        i += 4;
    }
    for (; i < len; ++i) shm_st1<POLICY>(dst + i, src[i]);
}

template <int U = 8, int POLICY = SHM_ST_STREAM>
__device__ __forceinline__ void shm_copy_coop(char *dst, const char *src, size_t n, unsigned tid, unsigned nthr)
{
    if (n == 0) return;
    size_t head = (16 - (reinterpret_cast<uintptr_t>(dst) & 15)) & 15;
    if (head > n) head = n;
    const size_t body = (n - head) & ~static_cast<size_t>(15);
    const size_t tail = n - head - body;
    if (nthr == 1) {              // a lone thread: pieces instead of bytes
        shm_copy_below16<POLICY>(dst, src, head);
        shm_copy_below16<POLICY>(dst + head + body, src + head + body, tail);
    } else {
        for (size_t i = tid; i < head; i += nthr) shm_st1<POLICY>(dst + i, src[i]);
        for (size_t i = tid; i < tail; i += nthr) shm_st1<POLICY>(dst + head + body + i, src[head + body + i]);
    }
    if (body == 0) return;
    shm_u32x4 *d = reinterpret_cast<shm_u32x4 *>(dst + head);
    const char *bs = src + head;
    const uint32_t mis = static_cast<uint32_t>(reinterpret_cast<uintptr_t>(bs) & 15);
    const size_t nvec = body >> 4;
    if (mis == 0) {
        shm_copy_body_aligned<U, POLICY>(d, reinterpret_cast<const shm_u32x4 *>(bs), nvec, tid, nthr);
        return;
    }
    const shm_u32x4 *sa = reinterpret_cast<const shm_u32x4 *>(bs - mis);
    const uint32_t sh = mis & 3;
    switch (mis >> 2) {       // uniform over the group: all threads share src and dst
    case 0: shm_copy_body_shifted<0, POLICY>(d, sa, nvec, sh, tid, nthr); break;
    case 1: shm_copy_body_shifted<1, POLICY>(d, sa, nvec, sh, tid, nthr); break;
    case 2: shm_copy_body_shifted<2, POLICY>(d, sa, nvec, sh, tid, nthr); break;
    default: shm_copy_body_shifted<3, POLICY>(d, sa, nvec, sh, tid, nthr); break;
    }
}

// ------------------------------------------------------------------------------------------
// Several work-groups sharing one message.  How the bytes are dealt to groups and lanes cannot be
// observed, so it is chosen for the memory system: on MI355X a wave sustains the highest HBM
// write rate when its successive 1 KiB accesses lie 32 KiB apart.  Up to 8 groups of 256 threads
// therefore form a "virtual block" whose 32 waves each own one 1 KiB column of a 32 KiB row; the
// virtual block walks tiles of U rows (256 KiB for U = 8), lane addresses advancing one row per
// unrolled access.  Vectors past the last whole tile are dealt 16 bytes per lane, round-robin
// over all groups.
// ------------------------------------------------------------------------------------------
struct shm_deal {
    size_t rowv;      // 16-byte vectors per row
    size_t tilev;     // vectors per tile (U rows)
    size_t ntiles;    // whole tiles in the message
    size_t vb, nvb;   // this group's virtual block, number of virtual blocks
    size_t col;       // this lane's vector within a row
    size_t rem_first; // first vector after the whole tiles
    size_t rem_lane;  // this lane's first remainder vector
    size_t rem_step;  // lanes in all groups together
};

// How many of the `nparts` groups take part in a message of nvec 16-byte vectors when every group is
// to get at least min_share bytes (0: all of them, the default).  A group's share has a fixed price
// when the group completes it by itself -- the drain of its stores and its part in the quiet that
// follows its put -- so a kernel that puts and then quiets in every group (shmx_putmem_parts followed
// by shmx_quiet_wg) passes SHM_MIN_SHARE_BYTES: beyond SHM_DEAL_ALWAYS_GROUPS groups the message is
// then dealt to further groups only while each still gets that much, and the others return at once,
// with nothing to complete.  Measured on MI355X (8 PEs, put + quiet inside a kernel of 1024 groups
// per PE): 16 MiB per PE 1.0 -> 1.9 TB/s, 32 MiB 1.0 -> 2.1 TB/s.  A put that the END of its kernel
// completes wants the opposite, every group at work (8 PEs x 8 MiB by 1024 groups each: 75 % of the
// HBM roofline against 54 % on 64 groups), hence the default.
constexpr size_t SHM_MIN_SHARE_BYTES = size_t(128) << 10;
constexpr unsigned SHM_DEAL_ALWAYS_GROUPS = 64;
__device__ __forceinline__ unsigned shm_deal_groups(size_t nvec, unsigned nparts, size_t min_share)
{
    if (min_share < 16 || nparts <= SHM_DEAL_ALWAYS_GROUPS) return nparts;
    size_t want = nvec / (min_share / 16);
    if (want < SHM_DEAL_ALWAYS_GROUPS) want = SHM_DEAL_ALWAYS_GROUPS;
    return want >= nparts ? nparts : static_cast<unsigned>(want & ~static_cast<size_t>(7));      // whole virtual blocks of 8
}

template <int U>
__device__ __forceinline__ shm_deal shm_deal_make(size_t nvec, unsigned part, unsigned nparts, unsigned tid, unsigned nthr)
{
    unsigned vw = nparts & (0u - nparts);      // largest power of two dividing nparts ...
    if (vw > 8) vw = 8;                        // ... capped at 8 groups = 32 KiB rows of 256-thread groups
    shm_deal d;
    d.rowv = static_cast<size_t>(vw) * nthr;
    d.tilev = d.rowv * U;
    d.ntiles = nvec / d.tilev;
    d.vb = part / vw;
    d.nvb = nparts / vw;
    d.col = static_cast<size_t>(part % vw) * nthr + tid;
    d.rem_first = d.ntiles * d.tilev;
    d.rem_lane = d.rem_first + static_cast<size_t>(part) * nthr + tid;
    d.rem_step = static_cast<size_t>(nparts) * nthr;
    return d;
}

// Whether group `part` moves any byte of an n-byte message dealt to `nparts` groups of `nthr`
// threads (a conservative test: true whenever one of its lanes could own a vector).
template <int U>
__device__ __forceinline__ bool shm_deal_has_share(size_t n, unsigned part, unsigned nparts, unsigned nthr, size_t min_share = 0)
{
    if (part == 0) return n != 0;
    nparts = shm_deal_groups(n >> 4, nparts, min_share);
    if (part >= nparts) return false;
    const shm_deal k = shm_deal_make<U>(n >> 4, part, nparts, 0, nthr);
    return k.vb < k.ntiles || k.rem_lane < ((n + 15) >> 4) + 1;
}

template <int U, int POLICY = SHM_ST_STREAM>
__device__ __forceinline__ void shm_copy_body_dealt(shm_u32x4 *d, const shm_u32x4 *s, size_t nvec, unsigned part,
                                                    unsigned nparts, unsigned tid, unsigned nthr)
{
    const shm_deal k = shm_deal_make<U>(nvec, part, nparts, tid, nthr);
    for (size_t t = k.vb; t < k.ntiles; t += k.nvb) {
        const size_t i = t * k.tilev + k.col;
        shm_u32x4 r[U];
#pragma unroll
        for (int u = 0; u < U; ++u) r[u] = shm_ld16(s + i + u * k.rowv);
#pragma unroll
        for (int u = 0; u < U; ++u) shm_st16<POLICY>(d + i + u * k.rowv, r[u]);
    }
    for (size_t i = k.rem_lane; i < nvec; i += 4 * k.rem_step) {
        shm_u32x4 r[4];
#pragma unroll
        for (int u = 0; u < 4; ++u)
            if (i + u * k.rem_step < nvec) r[u] = shm_ld16(s + i + u * k.rem_step);
#pragma unroll
        for (int u = 0; u < 4; ++u)
            if (i + u * k.rem_step < nvec) shm_st16<POLICY>(d + i + u * k.rem_step, r[u]);
    }
}

// Group `part` of `nparts` does its share of copying n bytes, any alignment.  All threads of all
// groups call this with the same dst/src/n.
constexpr size_t SHM_STORE_LINE = 1024, SHM_LINE_HEAD_MIN_BYTES = size_t(4) << 20;
template <int U = 8, int POLICY = SHM_ST_STREAM>
__device__ __forceinline__ void shm_copy_parts(char *dst, const char *src, size_t n, unsigned part, unsigned nparts, size_t min_share = 0)
{
    if (n == 0) return;
    const unsigned tid = threadIdx.x, nthr = blockDim.x;
    size_t head = (16 - (reinterpret_cast<uintptr_t>(dst) & 15)) & 15;
    if (head > n) head = n;
    const size_t body = (n - head) & ~static_cast<size_t>(15);
    const size_t tail = n - head - body;
    if (part == 0) {
        for (size_t i = tid; i < head; i += nthr) shm_st1<POLICY>(dst + i, src[i]);
        for (size_t i = tid; i < tail; i += nthr) shm_st1<POLICY>(dst + head + body + i, src[head + body + i]);
    }
    if (body == 0) return;
    shm_u32x4 *d = reinterpret_cast<shm_u32x4 *>(dst + head);
    const char *bs = src + head;
    const uint32_t mis = static_cast<uint32_t>(reinterpret_cast<uintptr_t>(bs) & 15);
    size_t nvec = body >> 4;
    nparts = shm_deal_groups(nvec, nparts, min_share);
    if (part >= nparts) return;
    // A message of SHM_LINE_HEAD_MIN_BYTES or more is dealt from where the destination reaches a multiple
    // of SHM_STORE_LINE bytes; the (fewer than 64) vectors before it are moved by the last group's first
    // lanes.  Stores that straddle lines are what costs (8 PEs x 24 MiB by 1024 groups each, % of the HBM
    // roofline: 74.6 on a boundary; destination 16 bytes past one 63.6 -> 72.9, both addresses 8 bytes past
    // 62.4 -> 74.2, 8 bytes apart 58.6 -> 67.9; 8 MiB: 58.1 -> 63.6, 56.1 -> 64.8, 59.4 -> 66.3; 4 MiB: both 8 bytes
    // past 52.6 -> 57.2; at 2 MiB and below the extra step of the last group costs what the boundary gains).
    if (nvec >= SHM_LINE_HEAD_MIN_BYTES / 16) {
        const size_t hv = ((SHM_STORE_LINE - (reinterpret_cast<uintptr_t>(d) & (SHM_STORE_LINE - 1))) & (SHM_STORE_LINE - 1)) >> 4;
        if (hv) {
            if (part == nparts - 1) shm_copy_coop<1, POLICY>(reinterpret_cast<char *>(d), bs, hv * 16, tid, nthr);
            d += hv, bs += hv * 16, nvec -= hv;
        }
    }
    if (mis == 0) {
        shm_copy_body_dealt<U, POLICY>(d, reinterpret_cast<const shm_u32x4 *>(bs), nvec, part, nparts, tid, nthr);
        return;
    }
    const shm_u32x4 *sa = reinterpret_cast<const shm_u32x4 *>(bs - mis);
    const uint32_t sh = mis & 3;
    const unsigned gtid = part * nthr + tid, gthr = nparts * nthr;
    switch (mis >> 2) {
    case 0: shm_copy_body_shifted<0, POLICY>(d, sa, nvec, sh, gtid, gthr); break;
    case 1: shm_copy_body_shifted<1, POLICY>(d, sa, nvec, sh, gtid, gthr); break;
    case 2: shm_copy_body_shifted<2, POLICY>(d, sa, nvec, sh, gtid, gthr); break;
    default: shm_copy_body_shifted<3, POLICY>(d, sa, nvec, sh, gtid, gthr); break;
    }
}

// ------------------------------------------------------------------------------------------
// Group-owned tiles: the dealing used for long messages.  A tile is U = 2 rows of 32 KiB and ONE
// group owns a whole tile: wave w walks the columns (1 KiB each) 8w..8w+7 (for 4 waves), its two
// accesses per column 32 KiB apart; group `part` takes tiles part, part + nparts, ...
//
// The order of the accesses is what decides the HBM rate, and what makes it depend -- or not -- on
// where source and destination lie relative to each other (the memory channels are chosen by a hash
// of the address, and a copy whose every wave reads X and writes X + delta at the same moment keeps
// read and write streams in a fixed relation for the whole launch: measured on MI355X, 8 PEs x
// 64-256 MiB, that form reaches 82 % of the HBM roofline for some placements and 70-75 % for others,
// e.g. with the destination 4 KiB or 1 MiB further on).  Two measures remove the dependence:
//   * a wave's stores trail its loads by LAG = 4 columns, continuously across the tiles the group
//     walks (eight loads in flight per lane instead of two), so that what a wave reads and what it
//     writes at one moment are 4 KiB apart in the message;
//   * group g starts its walk at column g mod 8 of each wave's eight, so that the groups running
//     at one moment do not all touch the same 1 KiB column of their 4 KiB blocks.
// With four tiles per group (the launcher's choice of grid) this form measures 79.8-80.9 % at
// 256 MiB x 8 PEs and 80.5-81.5 % at 64 MiB for every placement tried whose source is 64 KiB aligned
// (77-79 % otherwise); the per-column form it replaces measured 82 % at its best placement and 72-77 %
// at the others.  dst and src are 16-byte aligned, n is a multiple of 16.
// ------------------------------------------------------------------------------------------
// What a walk does with a column: copy it (the library's puts and gets), only read it, or only write
// it (the one-direction probes of the memory system, which must walk exactly as the copy does).
// `reg` is what a load leaves in a register slot until the store LAG columns later takes it.
struct shm_walk_copy {
    using reg = shm_u32x4;
    __device__ __forceinline__ reg load(const shm_u32x4 *p) const { return shm_ld16(p); }
    __device__ __forceinline__ void store(shm_u32x4 *p, reg v) { shm_st16(p, v); }
    __device__ __forceinline__ reg load_some(const shm_u32x4 *p) const { return load(p); }      // _some: any subset of lanes
    __device__ __forceinline__ void store_some(shm_u32x4 *p, reg v) { store(p, v); }
};
// The copy whose source lies W words and sh bytes (W, sh in 0..3, not both 0) beyond a 16-byte
// boundary: the walk is given that boundary as its source, every vector is put together from the two
// aligned words it straddles when it is stored (the word after the message's last vector holds at
// least one byte of the message, so it is mapped).
template <int W>
struct shm_walk_copy_shifted {
    struct reg {
        shm_u32x4 lo, hi;
    };
    uint32_t sh;
    // Whole columns (every lane of the wave at work, on consecutive vectors): the upper word of lane l
    // is the lower word of lane l + 1 and is taken from that lane's register when the column is stored;
    // lane 63 loads its own.  One load per vector and a one-lane load per wave instead of two loads per
    // vector: 8 PEs x 128 MiB with source and destination 3 or 8 bytes apart modulo 16, 74.2 -> 78.9 % of
    // the HBM roofline.
    __device__ __forceinline__ reg load(const shm_u32x4 *p) const
    {
        reg v;
        v.lo = shm_ld16(p);
        if ((threadIdx.x & 63) == 63) v.hi = shm_ld16(p + 1);
        return v;
    }
    __device__ __forceinline__ void store(shm_u32x4 *p, const reg &v)
    {
        shm_u32x4 hi;
        hi.x = __shfl_down(v.lo.x, 1), hi.y = __shfl_down(v.lo.y, 1), hi.z = __shfl_down(v.lo.z, 1), hi.w = __shfl_down(v.lo.w, 1);
        if ((threadIdx.x & 63) == 63) hi = v.hi;
        shm_st16(p, shm_realign<W>(v.lo, hi, sh));
    }
    // any subset of lanes (the partial tile)
    __device__ __forceinline__ reg load_some(const shm_u32x4 *p) const { return reg{shm_ld16(p), shm_ld16(p + 1)}; }
    __device__ __forceinline__ void store_some(shm_u32x4 *p, const reg &v) { shm_st16(p, shm_realign<W>(v.lo, v.hi, sh)); }
};
struct shm_walk_read {                 // the loads are folded into a word that the caller keeps alive
    using reg = shm_u32x4;
    uint32_t fold = 0;
    __device__ __forceinline__ reg load(const shm_u32x4 *p) const { return shm_ld16(p); }
    __device__ __forceinline__ void store(shm_u32x4 *, reg v) { fold ^= v.x ^ v.y ^ v.z ^ v.w; }
    __device__ __forceinline__ reg load_some(const shm_u32x4 *p) const { return load(p); }
    __device__ __forceinline__ void store_some(shm_u32x4 *p, reg v) { store(p, v); }
};
struct shm_walk_write {                // nothing is loaded: every store writes the pattern
    using reg = shm_u32x4;
    shm_u32x4 pattern;
    __device__ __forceinline__ reg load(const shm_u32x4 *) const { return pattern; }
    __device__ __forceinline__ void store(shm_u32x4 *p, reg v) { shm_st16(p, v); }
    __device__ __forceinline__ reg load_some(const shm_u32x4 *p) const { return load(p); }
    __device__ __forceinline__ void store_some(shm_u32x4 *p, reg v) { store(p, v); }
};

// One whole tile (or piece of a tile) of the walk: the stores of the columns loaded LAG steps ago,
// each followed by the load of the next column.  The first LAG of those stores belong to the
// previous tile, at `prev`; the FIRST tile of a walk has none (a compile-time case of its own: with
// a run-time flag the compiler peels the first tile itself and its copies of those loads lose the
// nontemporal hint, after which a repeated transfer finds an eighth of its source in the memory-side
// cache and measures 3-5 points more than a transfer of fresh data does).
template <int U, unsigned CPW, unsigned LAG, bool FIRST, typename OPS>
__device__ __forceinline__ void shm_tile_walk(OPS &ops, shm_u32x4 *d, const shm_u32x4 *s, size_t base, size_t prev, unsigned rot,
                                              typename OPS::reg (&r)[LAG][U])
{
    constexpr size_t rowv = 2048;                        // 32 KiB
    auto col = [&](unsigned c) { return static_cast<size_t>((c + rot) & (CPW - 1)) * 64; };
#pragma unroll
    for (unsigned c = 0; c < CPW; ++c) {
        const unsigned slot = c % LAG;                   // holds the column loaded LAG steps ago
        if (c >= LAG) {
#pragma unroll
            for (int u = 0; u < U; ++u) ops.store(d + base + col(c - LAG) + u * rowv, r[slot][u]);
        } else if (!FIRST) {
#pragma unroll
            for (int u = 0; u < U; ++u) ops.store(d + prev + col(c + CPW - LAG) + u * rowv, r[slot][u]);
        }
#pragma unroll
        for (int u = 0; u < U; ++u) r[slot][u] = ops.load(s + base + col(c) + u * rowv);
    }
}
// The stores still owed to the last whole tile of a walk.
template <int U, unsigned CPW, unsigned LAG, typename OPS>
__device__ __forceinline__ void shm_tile_walk_end(OPS &ops, shm_u32x4 *d, size_t prev, unsigned rot, typename OPS::reg (&r)[LAG][U])
{
    constexpr size_t rowv = 2048;
#pragma unroll
    for (unsigned c = CPW - LAG; c < CPW; ++c)
#pragma unroll
        for (int u = 0; u < U; ++u) ops.store(d + prev + static_cast<size_t>((c + rot) & (CPW - 1)) * 64 + u * rowv, r[c % LAG][u]);
}
// The last, partial tile of a message of nvec vectors: column by column, no lag.
template <int U, unsigned CPW, typename OPS>
__device__ __forceinline__ void shm_tile_partial(OPS &ops, shm_u32x4 *d, const shm_u32x4 *s, size_t base, size_t nvec)
{
    constexpr size_t rowv = 2048;
    for (unsigned c = 0; c < CPW; ++c) {
        const size_t i = base + static_cast<size_t>(c) * 64;
        typename OPS::reg q[U];
#pragma unroll
        for (int u = 0; u < U; ++u)
            if (i + u * rowv < nvec) q[u] = ops.load_some(s + i + u * rowv);
#pragma unroll
        for (int u = 0; u < U; ++u)
            if (i + u * rowv < nvec) ops.store_some(d + i + u * rowv, q[u]);
    }
}

template <int U, int NWAVES>
__device__ __forceinline__ void shm_copy_tiles_impl(char *dst, const char *src, size_t n, unsigned part, unsigned nparts)
{
    const shm_u32x4 *s = reinterpret_cast<const shm_u32x4 *>(src);
    shm_u32x4 *d = reinterpret_cast<shm_u32x4 *>(dst);
    const size_t nvec = n >> 4;
    constexpr size_t tilev = 2048 * U;                   // U rows of 32 KiB
    const size_t nwhole = nvec / tilev;                  // whole tiles; one more, partial, if nvec % tilev
    const unsigned wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    constexpr unsigned CPW = 32 / NWAVES;                // columns per wave; compile-time trip counts throughout
    constexpr unsigned LAG = CPW < 4 ? CPW : 4;
    static_assert(CPW % LAG == 0, "a register slot is refilled by the column LAG steps later, also across tiles");
    const unsigned rot = part & (CPW - 1);
    const size_t lane_off = static_cast<size_t>(wave * CPW) * 64 + lane;
    shm_walk_copy ops;
    if (part < nwhole) {
        shm_u32x4 r[LAG][U];
        size_t prev = part * tilev + lane_off;
        shm_tile_walk<U, CPW, LAG, true>(ops, d, s, prev, 0, rot, r);
        for (size_t t = part + nparts; t < nwhole; t += nparts) {
            const size_t base = t * tilev + lane_off;
            shm_tile_walk<U, CPW, LAG, false>(ops, d, s, base, prev, rot, r);
            prev = base;
        }
        shm_tile_walk_end<U, CPW, LAG>(ops, d, prev, rot, r);
    }
    if (nwhole * tilev < nvec && nwhole % nparts == part) shm_tile_partial<U, CPW>(ops, d, s, nwhole * tilev + lane_off, nvec);
}

// ------------------------------------------------------------------------------------------
// Tiles by ticket: the form of the long put.  The groups of a PE stay in the kernel and draw what
// they move next from a counter, in address order: a ticket is one of the PIECES equal parts of a
// 64 KiB tile (each wave's columns cut into PIECES runs; with 4 waves and PIECES = 2 a piece is 32 KiB:
// four columns of 1 KiB per wave in each of the tile's two rows), the partial tile at the end of the
// message is one ticket, the first.  Thread 0 draws the next number one piece ahead, so the atomic's latency is
// hidden behind the piece being moved, and hands it to the group through one of two LDS slots and one
// barrier per piece; the stores still trail the loads by LAG columns across pieces.  A group stops at
// the first number past the last piece.  With own_groups != 0 the first piece of group `part` is piece
// `part`, without a ticket (own_groups = number of groups drawing from this counter; tickets then
// start at that piece), which saves the one round trip nothing could hide.
// What it buys (measured on MI355X, puts of 32-256 MiB per PE, 4-8 PEs):
//   * what the chip touches at one moment is a compact window per PE that sweeps through the message
//     -- with 128 groups per PE and 32 KiB pieces, 4 MiB -- however unevenly the memory system serves
//     the groups; fixed shares drift apart and scatter the accesses;
//   * no group waits for work while another still has some: groups of one kernel are not served
//     equally (the ones started first are served first; with fixed shares half of a kernel's groups
//     finish in 200 us and the other half in 370-390 us), and the end of the transfer costs one
//     piece's time instead of one share's.
// 8 PEs x 128 groups, half-tile pieces: 84.1 % of the HBM roofline at 256 MiB per PE, 83.7 % at 128 MiB,
// 82.6 % at 64 MiB, within +-0.4 points over twelve random placements of the buffers (fixed tiles
// 77-79 %, fronts of 512 groups over 32 MiB segments 74-81 % depending on the placement); whole-tile
// pieces 81.1 / 80.7 / 79.7, quarter-tile pieces as half-tile ones; 112 or 144 groups per PE 81.6 %, 96
// or 192 81.5 %, 256 82.0 %: the window of 128 x 32 KiB = 4 MiB is the one this memory system likes.
// *counter must read first_ticket when the first group arrives and is left somewhere beyond the
// last ticket (every group that moved anything draws one ticket too many): whoever launches clears
// it, or the groups do (shm_tickets_done).  `part` also rotates the column walk.  dst and src 16-byte aligned, n a multiple of 16; every thread of the
// group calls.
// ------------------------------------------------------------------------------------------
template <int U, int NWAVES, int PIECES, typename OPS>
__device__ __forceinline__ void shm_walk_tiles_ticketed(OPS &ops, char *dst, const char *src, size_t n, unsigned part,
                                                        unsigned long long *counter, unsigned long long first_ticket, unsigned own_groups)
{
    __shared__ unsigned long long drawn[2];
    const shm_u32x4 *s = reinterpret_cast<const shm_u32x4 *>(src);
    shm_u32x4 *d = reinterpret_cast<shm_u32x4 *>(dst);
    const size_t nvec = n >> 4;
    constexpr size_t tilev = 2048 * U;
    const size_t nwhole = nvec / tilev;
    const size_t npieces = nwhole * PIECES, ntickets = npieces + (nwhole * tilev < nvec ? 1 : 0);
    const unsigned wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    constexpr unsigned CPW = 32 / NWAVES;                // a wave's columns in a whole tile
    constexpr unsigned CPP = CPW / PIECES;               // ... and in one piece
    static_assert(CPP >= 1 && CPP * PIECES == CPW, "whole columns per piece");
    constexpr unsigned LAG = CPP < 4 ? CPP : 4;
    static_assert(CPP % LAG == 0, "a register slot is refilled by the column LAG steps later, also across pieces");
    const unsigned rot = part & (CPP - 1);
    const size_t lane_off = static_cast<size_t>(wave * CPW) * 64 + lane;
    auto at = [&](size_t t) { return (t / PIECES) * tilev + (t % PIECES) * (CPP * 64) + lane_off; };
    auto draw = [&]() {
        return own_groups + __hip_atomic_fetch_add(counter, 1ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) - first_ticket;
    };
    typename OPS::reg r[LAG][U];
    size_t prev = 0;
    unsigned long long pending = 0;
    unsigned it = 0;
    // hands the number drawn during this piece to the group; two slots: the other one may still be being read
    auto next = [&]() {
        if (threadIdx.x == 0) drawn[(it + 1) & 1] = pending;
        __syncthreads();
        ++it;
        return static_cast<size_t>(drawn[it & 1]);
    };
    size_t t = part;
    if (own_groups == 0) {
        if (threadIdx.x == 0) drawn[0] = draw();
        __syncthreads();
        t = drawn[0];
    }
    // The partial tile at the end of the message is ticket 0 and the whole pieces follow it: one group
    // works through its predicated columns while the others have all their pieces before them.  As the
    // last ticket it was the last thing the kernel did, one group alone (8 PEs x 128 MiB less 112 bytes:
    // 80.2 % of the HBM roofline against 82.1 % for whole tiles).
    const size_t hp = ntickets - npieces;
    if (hp && t == 0) {
        if (threadIdx.x == 0) pending = draw();
        shm_tile_partial<U, CPW>(ops, d, s, nwhole * tilev + lane_off, nvec);
        t = next();
    }
    if (t < ntickets) {                                        // the walk's first piece has no stores owed
        if (threadIdx.x == 0) pending = draw();              // the next piece's number, on its way while this piece moves
        prev = at(t - hp);
        shm_tile_walk<U, CPP, LAG, true>(ops, d, s, prev, 0, rot, r);
        for (t = next(); t < ntickets; t = next()) {
            if (threadIdx.x == 0) pending = draw();
            const size_t base = at(t - hp);
            shm_tile_walk<U, CPP, LAG, false>(ops, d, s, base, prev, rot, r);
            prev = base;
        }
        shm_tile_walk_end<U, CPP, LAG>(ops, d, prev, rot, r);
    }
}
template <int U, int NWAVES, int PIECES = 2>
__device__ __forceinline__ void shm_copy_tiles_ticketed(char *dst, const char *src, size_t n, unsigned part, unsigned long long *counter,
                                                        unsigned long long first_ticket, unsigned own_groups = 0)
{
    shm_walk_copy ops;
    shm_walk_tiles_ticketed<U, NWAVES, PIECES>(ops, dst, src, n, part, counter, first_ticket, own_groups);
}
// The same for a source at any byte address (dst 16-byte aligned, n a multiple of 16).
template <int U, int NWAVES, int PIECES = 2>
__device__ __forceinline__ void shm_copy_tiles_ticketed_any(char *dst, const char *src, size_t n, unsigned part, unsigned long long *counter,
                                                            unsigned long long first_ticket, unsigned own_groups = 0)
{
    const uint32_t mis = static_cast<uint32_t>(reinterpret_cast<uintptr_t>(src) & 15);
    if (mis == 0) {
        shm_copy_tiles_ticketed<U, NWAVES, PIECES>(dst, src, n, part, counter, first_ticket, own_groups);
        return;
    }
    const char *sa = src - mis;
    switch (mis >> 2) {       // uniform over the grid
    case 0: {
        shm_walk_copy_shifted<0> ops{mis & 3};
        shm_walk_tiles_ticketed<U, NWAVES, PIECES>(ops, dst, sa, n, part, counter, first_ticket, own_groups);
    } break;
    case 1: {
        shm_walk_copy_shifted<1> ops{mis & 3};
        shm_walk_tiles_ticketed<U, NWAVES, PIECES>(ops, dst, sa, n, part, counter, first_ticket, own_groups);
    } break;
    case 2: {
        shm_walk_copy_shifted<2> ops{mis & 3};
        shm_walk_tiles_ticketed<U, NWAVES, PIECES>(ops, dst, sa, n, part, counter, first_ticket, own_groups);
    } break;
    default: {
        shm_walk_copy_shifted<3> ops{mis & 3};
        shm_walk_tiles_ticketed<U, NWAVES, PIECES>(ops, dst, sa, n, part, counter, first_ticket, own_groups);
    } break;
    }
}

// The drawing of tickets by itself, for kernels whose groups walk something other than a copy: group
// `part` of `groups` starts on number `part`; ahead() is called by every thread at the start of a
// piece (thread 0 draws the next number, which then travels while the piece is worked on) and next()
// at its end (the number is handed to the group through one of the two LDS words `slots`; one
// barrier).  The numbers drawn start at `groups`.
struct shm_ticket_draw {
    unsigned long long *counter;
    unsigned long long *slots;
    unsigned groups;
    unsigned it = 0;
    unsigned long long pending = 0;
    __device__ __forceinline__ void ahead()
    {
        if (threadIdx.x == 0) pending = groups + __hip_atomic_fetch_add(counter, 1ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    __device__ __forceinline__ size_t next()
    {
        if (threadIdx.x == 0) slots[(it + 1) & 1] = pending;
        __syncthreads();
        ++it;
        return static_cast<size_t>(slots[it & 1]);
    }
};

// A counter pair (ticket word, then a word that counts the groups that are through) that the last
// of `groups` groups to finish sets back to zero, so that the next launch -- or the next replay of
// a recorded one -- finds it as this one did.  Thread 0 of every group calls once, after its walk.
__device__ __forceinline__ void shm_tickets_done(unsigned long long *pair, unsigned groups)
{
    if (__hip_atomic_fetch_add(pair + 1, 1ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == groups - 1) {
        __hip_atomic_store(pair + 1, 0ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        __hip_atomic_store(pair, 0ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
}

template <int U = 2>
__device__ __forceinline__ void shm_copy_tiles(char *dst, const char *src, size_t n, unsigned part, unsigned nparts)
{
    switch (blockDim.x) {            // whole columns per wave need 1, 2, 4, 8 or 16 waves
    case 64: shm_copy_tiles_impl<U, 1>(dst, src, n, part, nparts); break;
    case 128: shm_copy_tiles_impl<U, 2>(dst, src, n, part, nparts); break;
    case 256: shm_copy_tiles_impl<U, 4>(dst, src, n, part, nparts); break;
    case 512: shm_copy_tiles_impl<U, 8>(dst, src, n, part, nparts); break;
    case 1024: shm_copy_tiles_impl<U, 16>(dst, src, n, part, nparts); break;
    default: shm_copy_parts<8, SHM_ST_STREAM>(dst, src, n, part, nparts); break;      // any other group size: the general dealing
    }
}

// ------------------------------------------------------------------------------------------
// RMA.  A put returns when the source may be reused; its bytes are delivered (visible to other
// PEs) after the caller's quiet.  A get returns with the bytes in place for the calling thread(s).
// Puts issued from inside a kernel choose their store policy by size.  Up to 64 bytes per
// participating thread they store write-through: the quiet that follows -- a full agent-scope
// release, so that the caller's own plain stores are covered as OpenSHMEM requires -- then finds
// no dirty lines of the put in the L2 and is several times cheaper, which is most of a small put's
// time (measured: 8 bytes by one group, put + quiet 0.69 -> 0.56 us).  Longer puts stream with
// nontemporal stores: a write-through store is acknowledged by memory rather than by the L2, and a
// few waves with a bounded number of stores in flight then move less than half the bytes per
// microsecond (1 MiB by one group: 17 us streaming, 38 us write-through).  Eight groups or more
// have the waves to cover that latency and store write-through up to 256 bytes per thread (put + quiet
// inside the kernel, 8 PEs x 64 groups: 2 MiB per PE 8.0 -> 4.4 us, 4 MiB 11.3 -> 8.0 us; at 1 KiB per
// thread 8 MiB 17.8 -> 19.6 us and 16 MiB 31 -> 39-44 us, and messages of 48 MiB and more move at 75 %
// of the HBM roofline written through against 81 % streamed).
// ------------------------------------------------------------------------------------------
constexpr size_t SHM_PUT_THROUGH_BYTES_PER_THREAD = 64;
constexpr size_t SHM_PUT_THROUGH_BYTES_PER_THREAD_MANY = 256;     // eight groups or more share the message

// Whether a put of n bytes by nparts groups of the calling group's size stores write-through (the
// rule of shm_put_parts / shm_put_coop): then nothing of it is dirty in the L2 afterwards and the
// plain group quiet, shmx_quiet_wg(), is the cheapest way to complete it.
__device__ __forceinline__ bool shm_put_stores_through(size_t n, unsigned nparts = 1, size_t min_share = 0);

template <int U>
__device__ __forceinline__ void shm_put_coop(char *dst, const char *src, size_t n, unsigned tid, unsigned nthr)
{
    if (n <= SHM_PUT_THROUGH_BYTES_PER_THREAD * nthr)
        shm_copy_coop<U, SHM_ST_THROUGH>(dst, src, n, tid, nthr);
    else
        shm_copy_coop<U, SHM_ST_STREAM>(dst, src, n, tid, nthr);
}
__device__ __forceinline__ bool shm_put_stores_through(size_t n, unsigned nparts, size_t min_share)
{
    const unsigned groups = shm_deal_groups(n >> 4, nparts, min_share);
    return n <= (groups >= 8 ? SHM_PUT_THROUGH_BYTES_PER_THREAD_MANY : SHM_PUT_THROUGH_BYTES_PER_THREAD) * blockDim.x * groups;
}
template <int U>
__device__ __forceinline__ void shm_put_parts(char *dst, const char *src, size_t n, unsigned part, unsigned nparts, size_t min_share = 0)
{
    if (shm_put_stores_through(n, nparts, min_share))
        shm_copy_parts<U, SHM_ST_THROUGH>(dst, src, n, part, nparts, min_share);
    else
        shm_copy_parts<U, SHM_ST_STREAM>(dst, src, n, part, nparts, min_share);
}

// Scalar put and get (paper section "Remote Memory Access": the ishmem_long_p example -- translate
// the symmetric address, then one store).  T is any 1-, 2-, 4- or 8-byte trivially copyable type.
// p returns at once and is delivered after quiet; the store is write-through so that the quiet is
// cheap.  g returns the remote element's current value (read at agent scope, past this compute
// unit's cache).
template <typename T>
__device__ __forceinline__ void shm_p(const shm_dev_ctx &c, uint64_t dst_off, T value, int pe)
{
    static_assert(sizeof(T) == 1 || sizeof(T) == 2 || sizeof(T) == 4 || sizeof(T) == 8, "scalar put/get moves 1, 2, 4 or 8 bytes");
    T *d = reinterpret_cast<T *>(shm_ptr(c, dst_off, pe));
    if constexpr (sizeof(T) == 8) {
        uint64_t bits;
        __builtin_memcpy(&bits, &value, 8);
        __hip_atomic_store(reinterpret_cast<uint64_t *>(d), bits, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    } else if constexpr (sizeof(T) == 4) {
        uint32_t bits;
        __builtin_memcpy(&bits, &value, 4);
        __hip_atomic_store(reinterpret_cast<uint32_t *>(d), bits, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    } else {
        *d = value;       // sub-word stores have no agent-scope spelling; quiet's release covers them
    }
}
template <typename T>
__device__ __forceinline__ T shm_g(const shm_dev_ctx &c, uint64_t src_off, int pe)
{
    static_assert(sizeof(T) == 1 || sizeof(T) == 2 || sizeof(T) == 4 || sizeof(T) == 8, "scalar put/get moves 1, 2, 4 or 8 bytes");
    const T *s = reinterpret_cast<const T *>(shm_ptr(c, src_off, pe));
    T value;
    if constexpr (sizeof(T) == 8) {
        const uint64_t bits = __hip_atomic_load(reinterpret_cast<const uint64_t *>(s), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        __builtin_memcpy(&value, &bits, 8);
    } else if constexpr (sizeof(T) == 4) {
        const uint32_t bits = __hip_atomic_load(reinterpret_cast<const uint32_t *>(s), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        __builtin_memcpy(&value, &bits, 4);
    } else {
        value = __builtin_nontemporal_load(s);
    }
    return value;
}

// Single-thread forms.  One lane's bandwidth is (bytes in flight) / (memory latency), so U, the
// number of 16-byte loads issued before the first store, is what a caller with registers to spare
// can raise (at most 63 loads can be outstanding per wave).
template <int U = 4>
__device__ __forceinline__ void shm_putmem(const shm_dev_ctx &c, int me, uint64_t dst_off, uint64_t src_off, size_t n, int pe)
{
    shm_put_coop<U>(shm_ptr(c, dst_off, pe), shm_ptr(c, src_off, me), n, 0, 1);
}
template <int U = 4>
__device__ __forceinline__ void shm_getmem(const shm_dev_ctx &c, int me, uint64_t dst_off, uint64_t src_off, size_t n, int pe)
{
    shm_copy_coop<U>(shm_ptr(c, dst_off, me), shm_ptr(c, src_off, pe), n, 0, 1);
}

// Sub-group (wave64) forms: the 64 lanes of the calling wave share the copy.
__device__ __forceinline__ void shmx_putmem_wave(const shm_dev_ctx &c, int me, uint64_t dst_off, uint64_t src_off, size_t n, int pe)
{
    shm_put_coop<8>(shm_ptr(c, dst_off, pe), shm_ptr(c, src_off, me), n, __lane_id(), 64);
}
__device__ __forceinline__ void shmx_getmem_wave(const shm_dev_ctx &c, int me, uint64_t dst_off, uint64_t src_off, size_t n, int pe)
{
    shm_copy_coop<8>(shm_ptr(c, dst_off, me), shm_ptr(c, src_off, pe), n, __lane_id(), 64);
}

// Work-group forms (paper section "Proposed Device APIs").  The entry barrier makes every
// thread's earlier writes to the source part of the message; the exit barrier lets any thread
// reuse the source (put) or read the destination (get) on return.
__device__ __forceinline__ void shmx_putmem_wg(const shm_dev_ctx &c, int me, uint64_t dst_off, uint64_t src_off, size_t n, int pe)
{
    __syncthreads();
    shm_put_parts<8>(shm_ptr(c, dst_off, pe), shm_ptr(c, src_off, me), n, 0, 1);
    __syncthreads();
}
__device__ __forceinline__ void shmx_getmem_wg(const shm_dev_ctx &c, int me, uint64_t dst_off, uint64_t src_off, size_t n, int pe)
{
    __syncthreads();
    shm_copy_parts<8>(shm_ptr(c, dst_off, me), shm_ptr(c, src_off, pe), n, 0, 1);
    __syncthreads();
}

// The same for `nparts` work-groups of one PE sharing one message; this group is number `part`.
// Every thread of every group passes the same offsets and n.  On return this group's share is
// done; the message is complete when all groups have returned (and delivered after their quiet).
// min_share: see shm_deal_groups (a kernel whose groups each quiet after the put passes
// SHM_MIN_SHARE_BYTES and asks shm_deal_has_share, with the same value, which groups have anything to
// complete).
__device__ __forceinline__ void shmx_putmem_parts(const shm_dev_ctx &c, int me, uint64_t dst_off, uint64_t src_off, size_t n,
                                                  int pe, unsigned part, unsigned nparts, size_t min_share = 0)
{
    __syncthreads();
    shm_put_parts<8>(shm_ptr(c, dst_off, pe), shm_ptr(c, src_off, me), n, part, nparts, min_share);
    __syncthreads();
}
__device__ __forceinline__ void shmx_getmem_parts(const shm_dev_ctx &c, int me, uint64_t dst_off, uint64_t src_off, size_t n,
                                                  int pe, unsigned part, unsigned nparts)
{
    __syncthreads();
    shm_copy_parts<8>(shm_ptr(c, dst_off, me), shm_ptr(c, src_off, pe), n, part, nparts);
    __syncthreads();
}

// The same with group-owned tiles (see shm_copy_tiles): for long messages.  Offsets 16-byte aligned;
// the last n mod 16 bytes are copied by group 0.  NWAVES != 0 states the group size at compile time
// (64 * NWAVES work-items; the library's own kernels do), 0 takes it from blockDim.
template <int NWAVES = 0>
__device__ __forceinline__ void shmx_copy_tiles_wg(char *d, const char *s, size_t n, unsigned part, unsigned nparts)
{
    __syncthreads();
    const size_t body = n & ~static_cast<size_t>(15);
    if (NWAVES)
        shm_copy_tiles_impl<2, NWAVES ? NWAVES : 1>(d, s, body, part, nparts);
    else
        shm_copy_tiles<2>(d, s, body, part, nparts);
    if (part == 0)
        for (size_t i = body + threadIdx.x; i < n; i += blockDim.x) d[i] = s[i];
    __syncthreads();
}
template <int NWAVES = 0>
__device__ __forceinline__ void shmx_putmem_tiles(const shm_dev_ctx &c, int me, uint64_t dst_off, uint64_t src_off, size_t n, int pe,
                                                  unsigned part, unsigned nparts)
{
    shmx_copy_tiles_wg<NWAVES>(shm_ptr(c, dst_off, pe), shm_ptr(c, src_off, me), n, part, nparts);
}
template <int NWAVES = 0>
__device__ __forceinline__ void shmx_getmem_tiles(const shm_dev_ctx &c, int me, uint64_t dst_off, uint64_t src_off, size_t n, int pe,
                                                  unsigned part, unsigned nparts)
{
    shmx_copy_tiles_wg<NWAVES>(shm_ptr(c, dst_off, me), shm_ptr(c, src_off, pe), n, part, nparts);
}

// A long put shared by groups that draw what they move from a ticket counter (shm_copy_tiles_ticketed):
// for groups that stay in the kernel.  `counter` is a 64-bit word in device memory that reads
// first_ticket before the first group arrives; own_groups: 0, or the number of groups that draw from
// it, group `part` of them then starting on piece `part` without a ticket.  NWAVES states the group size
// (64 * NWAVES work-items).  Offsets 16-byte aligned; the last n mod 16 bytes are copied by group 0.
template <int NWAVES>
__device__ __forceinline__ void shmx_putmem_tickets(const shm_dev_ctx &c, int me, uint64_t dst_off, uint64_t src_off, size_t n, int pe,
                                                    unsigned part, unsigned long long *counter, unsigned long long first_ticket,
                                                    unsigned own_groups = 0)
{
    char *d = shm_ptr(c, dst_off, pe);
    const char *s = shm_ptr(c, src_off, me);
    __syncthreads();
    const size_t body = n & ~static_cast<size_t>(15);
    shm_copy_tiles_ticketed<2, NWAVES>(d, s, body, part, counter, first_ticket, own_groups);
    if (part == 0)
        for (size_t i = body + threadIdx.x; i < n; i += blockDim.x) d[i] = s[i];
    __syncthreads();
}

// ------------------------------------------------------------------------------------------
// Ordering.  All logical PEs live on one GPU, so agent scope is the widest scope ever needed
// between PEs.  quiet = the calling thread's puts and atomics are complete and visible to every
// PE; fence = they are ordered before its later ones (same instruction here).
// ------------------------------------------------------------------------------------------
__device__ __forceinline__ void shm_quiet() { __builtin_amdgcn_fence(__ATOMIC_RELEASE, "agent"); }
__device__ __forceinline__ void shm_fence() { __builtin_amdgcn_fence(__ATOMIC_RELEASE, "agent"); }
// Group form: after the barrier every thread's stores happen before the leader's agent-scope
// release, so one cache write-back per group (not one per wave) completes the group's puts.
__device__ __forceinline__ void shmx_quiet_wg()
{
    __syncthreads();
    if (threadIdx.x == 0) __builtin_amdgcn_fence(__ATOMIC_RELEASE, "agent");
    __syncthreads();
}

// The same for grids of many groups.  An agent-scope release is one write-back of the XCD's whole
// L2 (buffer_wbl2), and the write-backs of one XCD are served one after another at a quarter to
// half a microsecond each, dirty lines or not: a grid whose every group releases for itself pays
// (groups per XCD) x that, which is most of the time of a put followed by its quiet once a grid has
// hundreds of groups.  But ONE write-back covers every store that had reached that L2 when it
// began, whoever issued it.  So the groups of an XCD share their releases through one 64-bit word
// per XCD (in the library's tail of PE 0's partition; the XCD number is the hardware's XCC_ID
// register) by the protocol of shm_release_algo.hpp.  Every wave first waits for the
// acknowledgement of its own stores (s_waitcnt vmcnt(0): they are in the L2 or beyond); then the
// group's leader runs the protocol.  Small grids (fewer than SHMD_QUIET_SHARED_MIN_GROUPS groups)
// release directly: an atomic costs more than a write-back nobody queues for.
#define SHMD_INTERNAL_QUIET 33280u            // 8 words, 128 bytes apart
#define SHMD_INTERNAL_TICKETS 36864u          // SHMD_TICKET_WORDS uint64 in every partition's tail: ticket counters of the long puts
#define SHMD_TICKET_WORDS 512u
#define SHMD_TICKET_TIMED_WORDS 504u          // words 0..503: the timed put, one per repetition (cleared by its launcher)
#define SHMD_TICKET_TEAM 504u                 // a counter pair (ticket, groups through) for team puts and gets ...
#define SHMD_TICKET_COLL 506u                 // ... for team collectives ...
#define SHMD_TICKET_PROBE 508u                // ... for the stream probes ...
#define SHMD_TICKET_PE 510u                   // ... and for a PE's own long puts and gets; the pairs reset themselves (shm_tickets_done)
// A walk in several ways (the message cut into that many runs of whole tiles, each with its own groups
// and its own counter pair) keeps its pairs SHMD_TICKET_WAY_BYTES apart: tickets are drawn with an
// atomic on one word, the memory side performs the atomics on one line -- and on neighbouring lines --
// one after another (some 60 million a second), and one walk that moves 3 TB/s in 32 KiB pieces draws
// 100 million.
#define SHMD_INTERNAL_WAY_TICKETS 40960u      // SHMD_TICKET_MAX_WAYS pairs, SHMD_TICKET_WAY_BYTES apart: a PE's own long puts and gets in ways
#define SHMD_TICKET_WAY_BYTES 4096u
#define SHMD_TICKET_MAX_WAYS 4u
#define SHMD_QUIET_SHARED_MIN_GROUPS 64u
#define SHMD_QUIET_SPIN_LIMIT 4096

__device__ __forceinline__ unsigned shm_xcc_id()
{
    unsigned v;
    asm volatile("s_getreg_b32 %0, hwreg(HW_REG_XCC_ID)" : "=s"(v));
    return v & 7u;
}

struct shm_release_device_ops {
    unsigned long long *word;
    __device__ __forceinline__ unsigned long long fetch_or_lock() { return __hip_atomic_fetch_or(word, 1ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }
    __device__ __forceinline__ unsigned long long load() { return __hip_atomic_load(word, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }
    __device__ __forceinline__ void store(unsigned long long v) { __hip_atomic_store(word, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }
    __device__ __forceinline__ void write_back() { __builtin_amdgcn_fence(__ATOMIC_RELEASE, "agent"); }      // the write-back, waited for
    __device__ __forceinline__ void pause() { __builtin_amdgcn_s_sleep(2); }
};

// One thread; the stores it speaks for are acknowledged.
__device__ __forceinline__ void shm_release_shared(const shm_dev_ctx &c)
{
    shm_release_device_ops ops{reinterpret_cast<unsigned long long *>(c.base[0] + c.internal_off + SHMD_INTERNAL_QUIET + 128u * shm_xcc_id())};
    shm_release_shared_algo(ops, SHMD_QUIET_SPIN_LIMIT);
}

// bulk == false says that the group's puts since its last quiet all stored write-through
// (shm_put_stores_through): a release then finds nothing of them dirty and costs a quarter of a
// microsecond, less than the atomic the shared form starts with (measured, 64-256 groups of one PE
// putting 4-16 KiB each and quieting: 2.5-2.8 us directly, 3.2-4.5 us shared; with 64 KiB or more
// per group the shared form wins, 11.0 against 15.6 us for 64 groups and more with more groups).
__device__ __forceinline__ void shmx_quiet_wg(const shm_dev_ctx &c, bool bulk = true)
{
    if (!bulk || gridDim.x * gridDim.y * gridDim.z < SHMD_QUIET_SHARED_MIN_GROUPS) {
        shmx_quiet_wg();
        return;
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");      // this wave's stores have reached the L2
    __syncthreads();                                      // ... and so have every other wave's of the group
    if (threadIdx.x == 0) shm_release_shared(c);
    __syncthreads();
}

// ------------------------------------------------------------------------------------------
// Signals: 64-bit unsigned words on the symmetric heap.
// ------------------------------------------------------------------------------------------
__device__ __forceinline__ void shm_signal_update(uint64_t *sig, uint64_t v, int op)
{
    if (op == SHMD_SIGNAL_SET)
        __hip_atomic_store(sig, v, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_AGENT);
    else
        __hip_atomic_fetch_add(sig, v, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_AGENT);
}

__device__ __forceinline__ uint64_t shm_signal_fetch(const shm_dev_ctx &c, int me, uint64_t sig_off)
{
    return __hip_atomic_load(reinterpret_cast<uint64_t *>(shm_ptr(c, sig_off, me)), __ATOMIC_ACQUIRE,
                             __HIP_MEMORY_SCOPE_AGENT);
}

__device__ __forceinline__ bool shm_cmp(uint64_t a, int cmp, uint64_t b)
{
    switch (cmp) {
    case SHMD_CMP_EQ: return a == b;
    case SHMD_CMP_NE: return a != b;
    case SHMD_CMP_GT: return a > b;
    case SHMD_CMP_GE: return a >= b;
    case SHMD_CMP_LT: return a < b;
    default: return a <= b;
    }
}

// Spin until cmp(signal, val) holds; acquire.  Bounded: after wait_ticks the status word
// is set and the call returns the last value read, so a kernel can never hang on a signal that
// is not coming.
__device__ __forceinline__ uint64_t shm_signal_wait_until(const shm_dev_ctx &c, int me, uint64_t sig_off, int cmp, uint64_t val)
{
    uint64_t *sig = reinterpret_cast<uint64_t *>(shm_ptr(c, sig_off, me));
    const uint64_t t0 = wall_clock64();
    uint64_t cur;
    for (;;) {
        cur = __hip_atomic_load(sig, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if (shm_cmp(cur, cmp, val)) break;
        if (wall_clock64() - t0 > c.wait_ticks) {
            __hip_atomic_store(c.status, 1ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
            break;
        }
        __builtin_amdgcn_s_sleep(2);
    }
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
    return cur;
}

// Work-group form: one thread polls (the paper's leader-thread pattern) and acquires at agent
// scope; the value is shared through LDS, and the barrier extends the leader's acquire to the whole
// group (all waves of a work-group share one CU's vector cache, which the leader has invalidated).
__device__ __forceinline__ uint64_t shmx_signal_wait_until_wg(const shm_dev_ctx &c, int me, uint64_t sig_off, int cmp, uint64_t val)
{
    __shared__ uint64_t seen;
    if (threadIdx.x == 0) seen = shm_signal_wait_until(c, me, sig_off, cmp, val);
    __syncthreads();
    const uint64_t v = seen;
    __syncthreads();          // `seen` may be overwritten by the next wait only after everyone read it
    return v;
}

// ------------------------------------------------------------------------------------------
// Point-to-point synchronisation on 64-bit signed variables of the caller's own heap (paper section
// "Proposed Device APIs": these routines are callable from the device; semantics of OpenSHMEM 1.5
// wait_until / test and their all / any / some forms).  Comparisons are SIGNED here (signals compare
// unsigned).  `status`, if not null, has one int per variable; a nonzero entry takes that variable
// out of the set.  Waits are bounded like every wait of the library.  Called by ONE thread.
// ------------------------------------------------------------------------------------------
#define SHMD_NO_INDEX (~static_cast<size_t>(0))

__device__ __forceinline__ bool shm_cmp_i64(int64_t a, int cmp, int64_t b)
{
    switch (cmp) {
    case SHMD_CMP_EQ: return a == b;
    case SHMD_CMP_NE: return a != b;
    case SHMD_CMP_GT: return a > b;
    case SHMD_CMP_GE: return a >= b;
    case SHMD_CMP_LT: return a < b;
    default: return a <= b;
    }
}

__device__ __forceinline__ int64_t shm_ivar_load(const shm_dev_ctx &c, int me, uint64_t off, size_t i)
{
    return __hip_atomic_load(reinterpret_cast<const int64_t *>(shm_ptr(c, off, me)) + i, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// One look at every selected variable.  Returns how many satisfy the comparison; writes their indices
// to `indices` (if not null) and the first of them to *first.
__device__ __forceinline__ size_t shm_test_scan(const shm_dev_ctx &c, int me, uint64_t off, size_t n, const int *status, int cmp,
                                                int64_t val, size_t *indices, size_t *first, size_t *selected)
{
    size_t hits = 0, sel = 0;
    *first = SHMD_NO_INDEX;
    for (size_t i = 0; i < n; ++i) {
        if (status != nullptr && status[i] != 0) continue;
        ++sel;
        if (shm_cmp_i64(shm_ivar_load(c, me, off, i), cmp, val)) {
            if (hits == 0) *first = i;
            if (indices != nullptr) indices[hits] = i;
            ++hits;
        }
    }
    *selected = sel;
    return hits;
}

// test: true (with acquire) if the comparison holds now.
__device__ __forceinline__ bool shm_test(const shm_dev_ctx &c, int me, uint64_t off, int cmp, int64_t val)
{
    const bool ok = shm_cmp_i64(shm_ivar_load(c, me, off, 0), cmp, val);
    if (ok) __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
    return ok;
}

// wait_until: spins until the comparison holds; returns the satisfying value.
__device__ __forceinline__ int64_t shm_wait_until(const shm_dev_ctx &c, int me, uint64_t off, int cmp, int64_t val)
{
    const uint64_t t0 = wall_clock64();
    int64_t cur;
    for (;;) {
        cur = shm_ivar_load(c, me, off, 0);
        if (shm_cmp_i64(cur, cmp, val)) break;
        if (wall_clock64() - t0 > c.wait_ticks) {
            __hip_atomic_store(c.status, 1ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
            break;
        }
        __builtin_amdgcn_s_sleep(2);
    }
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
    return cur;
}

// The set forms.  need_all: every selected variable must satisfy (all), else at least one (any / some).
// Returns the number of satisfying variables at the moment the condition was met (0 only if nothing is
// selected or the wait ran into its bound); *first and indices as in shm_test_scan.
__device__ __forceinline__ size_t shm_wait_until_set(const shm_dev_ctx &c, int me, uint64_t off, size_t n, const int *status, int cmp,
                                                     int64_t val, bool need_all, size_t *indices, size_t *first)
{
    const uint64_t t0 = wall_clock64();
    size_t hits, selected;
    for (;;) {
        hits = shm_test_scan(c, me, off, n, status, cmp, val, indices, first, &selected);
        if (selected == 0 || (need_all ? hits == selected : hits > 0)) break;
        if (wall_clock64() - t0 > c.wait_ticks) {
            __hip_atomic_store(c.status, 1ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
            hits = 0;
            break;
        }
        __builtin_amdgcn_s_sleep(2);
    }
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
    return hits;
}
__device__ __forceinline__ void shm_wait_until_all(const shm_dev_ctx &c, int me, uint64_t off, size_t n, const int *status, int cmp, int64_t val)
{
    size_t first;
    (void)shm_wait_until_set(c, me, off, n, status, cmp, val, true, nullptr, &first);
}
// Index of one satisfying variable, SHMD_NO_INDEX if none is selected.
__device__ __forceinline__ size_t shm_wait_until_any(const shm_dev_ctx &c, int me, uint64_t off, size_t n, const int *status, int cmp, int64_t val)
{
    size_t first;
    (void)shm_wait_until_set(c, me, off, n, status, cmp, val, false, nullptr, &first);
    return first;
}
// Number of satisfying variables (at least one unless none is selected); their indices to `indices`.
__device__ __forceinline__ size_t shm_wait_until_some(const shm_dev_ctx &c, int me, uint64_t off, size_t n, size_t *indices, const int *status,
                                                      int cmp, int64_t val)
{
    size_t first;
    return shm_wait_until_set(c, me, off, n, status, cmp, val, false, indices, &first);
}
// The non-blocking forms: one scan, acquire when the answer is positive.
__device__ __forceinline__ bool shm_test_all(const shm_dev_ctx &c, int me, uint64_t off, size_t n, const int *status, int cmp, int64_t val)
{
    size_t first, selected;
    const size_t hits = shm_test_scan(c, me, off, n, status, cmp, val, nullptr, &first, &selected);
    const bool ok = hits == selected;              // an empty set is trivially satisfied
    if (ok) __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
    return ok;
}
__device__ __forceinline__ size_t shm_test_any(const shm_dev_ctx &c, int me, uint64_t off, size_t n, const int *status, int cmp, int64_t val)
{
    size_t first, selected;
    if (shm_test_scan(c, me, off, n, status, cmp, val, nullptr, &first, &selected) > 0) __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
    return first;
}
__device__ __forceinline__ size_t shm_test_some(const shm_dev_ctx &c, int me, uint64_t off, size_t n, size_t *indices, const int *status,
                                                int cmp, int64_t val)
{
    size_t first, selected;
    const size_t hits = shm_test_scan(c, me, off, n, status, cmp, val, indices, &first, &selected);
    if (hits > 0) __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
    return hits;
}

// Put with signal for one work-group, or for `nparts` work-groups sharing one message.
//
// OpenSHMEM orders the signal after THIS put's payload only (earlier puts need fence/quiet), so a
// full agent-scope release -- whose cache write-back costs about a quarter of a microsecond and
// serialises over every group of an XCD -- is not required, only that the payload is performed at
// agent scope before the signal is.  That is arranged directly: every payload store is written
// through the XCD's L2 (sc1, the encoding of an agent-scope atomic store), every wave waits for the
// acknowledgement of its own stores (s_waitcnt vmcnt(0): for a store of that scope the
// acknowledgement means it is performed at agent scope), the group barrier collects the waves, and
// only then does the leader touch the arrival counter and the signal, with relaxed agent-scope
// atomics.  Group `part` copies its share; the group whose arrival completes the message (counted
// in *arrive, which it resets to zero) updates the signal.  With nparts == 1 the counter is not
// touched and may be null.  (SHMD_ARRIVE_ORDER / SHMD_SIGNAL_ORDER: relaxed here, release/acquire in
// the cross-check build.)
__device__ __forceinline__ void shmx_putmem_signal_parts(const shm_dev_ctx &c, int me, uint64_t dst_off, uint64_t src_off,
                                                         size_t n, uint64_t sig_off, uint64_t sig_val, int sig_op, int pe,
                                                         uint64_t *arrive, unsigned part, unsigned nparts)
{
    constexpr int arrive_order = SHMD_ARRIVE_ORDER, signal_order = SHMD_SIGNAL_ORDER;
    __syncthreads();
    shm_copy_parts<8, SHM_ST_THROUGH>(shm_ptr(c, dst_off, pe), shm_ptr(c, src_off, me), n, part, nparts);
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");     // this wave's payload is performed at agent scope
    __syncthreads();                                      // ... and so is every other wave's of the group
    if (threadIdx.x == 0) {
        bool last = true;
        if (nparts > 1) {
            const uint64_t old = __hip_atomic_fetch_add(arrive, 1ull, arrive_order, __HIP_MEMORY_SCOPE_AGENT);
            last = (old == nparts - 1);
            if (last) __hip_atomic_store(arrive, 0ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
        if (last) {
            uint64_t *sig = reinterpret_cast<uint64_t *>(shm_ptr(c, sig_off, pe));
            if (sig_op == SHMD_SIGNAL_SET)
                __hip_atomic_store(sig, sig_val, signal_order, __HIP_MEMORY_SCOPE_AGENT);
            else
                __hip_atomic_fetch_add(sig, sig_val, signal_order, __HIP_MEMORY_SCOPE_AGENT);
        }
    }
}

__device__ __forceinline__ void shmx_putmem_signal_wg(const shm_dev_ctx &c, int me, uint64_t dst_off, uint64_t src_off, size_t n,
                                                      uint64_t sig_off, uint64_t sig_val, int sig_op, int pe)
{
    shmx_putmem_signal_parts(c, me, dst_off, src_off, n, sig_off, sig_val, sig_op, pe, nullptr, 0, 1);
}

// ------------------------------------------------------------------------------------------
// 64-bit atomics on any PE's heap (paper section "Proposed Device APIs": scalar, no group form).
// Relaxed, agent scope; order them with shm_fence/shm_quiet like any other operation.
// ------------------------------------------------------------------------------------------
__device__ __forceinline__ int64_t *shm_i64(const shm_dev_ctx &c, uint64_t off, int pe)
{
    return reinterpret_cast<int64_t *>(shm_ptr(c, off, pe));
}
__device__ __forceinline__ int64_t shm_atomic_fetch(const shm_dev_ctx &c, uint64_t off, int pe)
{
    return __hip_atomic_load(shm_i64(c, off, pe), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void shm_atomic_set(const shm_dev_ctx &c, uint64_t off, int64_t v, int pe)
{
    __hip_atomic_store(shm_i64(c, off, pe), v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ int64_t shm_atomic_swap(const shm_dev_ctx &c, uint64_t off, int64_t v, int pe)
{
    return __hip_atomic_exchange(shm_i64(c, off, pe), v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ int64_t shm_atomic_compare_swap(const shm_dev_ctx &c, uint64_t off, int64_t cond, int64_t v, int pe)
{
    int64_t expected = cond;
    __hip_atomic_compare_exchange_strong(shm_i64(c, off, pe), &expected, v, __ATOMIC_RELAXED, __ATOMIC_RELAXED,
                                         __HIP_MEMORY_SCOPE_AGENT);
    return expected;      // the value found: equals cond exactly when the swap happened
}
__device__ __forceinline__ int64_t shm_atomic_fetch_add(const shm_dev_ctx &c, uint64_t off, int64_t v, int pe)
{
    return __hip_atomic_fetch_add(shm_i64(c, off, pe), v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void shm_atomic_add(const shm_dev_ctx &c, uint64_t off, int64_t v, int pe)
{
    (void)__hip_atomic_fetch_add(shm_i64(c, off, pe), v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ int64_t shm_atomic_fetch_inc(const shm_dev_ctx &c, uint64_t off, int pe)
{
    return shm_atomic_fetch_add(c, off, 1, pe);
}
__device__ __forceinline__ void shm_atomic_inc(const shm_dev_ctx &c, uint64_t off, int pe) { shm_atomic_add(c, off, 1, pe); }

// Fetch-and-increment in batches by one work-group, on a symmetric table of n_ctr int64 counters
// per PE.  The paper (section "Proposed Device APIs") gives the atomics no group form because on its
// hardware scalar operations gain nothing from one; on this GPU the memory-side atomic units
// (about 12 G operations per second for the whole chip) are the limit of a storm of scalar
// fetch-adds, and a group that counts its own increments in LDS first sends one fetch-add per
// counter it touched instead of one per increment -- from consecutive lanes to consecutive
// counters, so that a wave's 64 atomics fall on eight 64-byte lines.
//
// Every thread of the group calls this.  count_each(visit) calls visit(id) once for each of the
// thread's increments (id = pe * n_ctr + index; any number of them, none included);
// fetch_each(visit) walks the same increments again, and there visit(id) returns the value that
// increment fetched.  Three steps: the increments are counted per counter in `table`; each touched
// entry is replaced by what ONE global fetch-add of its count returns; the second walk increments
// the entries again, now with return.  The values are those of one valid serialisation: the
// group's increments of a counter take consecutive places in that counter's order.  `table` is
// LDS, npes * n_ctr entries of 8 bytes, owned by the call from entry to return.  Relaxed, agent
// scope, like the scalar atomics.
template <typename CountEach, typename FetchEach>
__device__ __forceinline__ void shmx_atomic_fetch_inc_batch_wg(const shm_dev_ctx &c, uint64_t ctr_off, uint32_t n_ctr,
                                                               unsigned long long *table, CountEach count_each, FetchEach fetch_each)
{
    const uint32_t entries = static_cast<uint32_t>(c.npes) * n_ctr;
    for (uint32_t e = threadIdx.x; e < entries; e += blockDim.x) table[e] = 0;
    __syncthreads();
    count_each([&](uint32_t id) { (void)atomicAdd(table + id, 1ull); });
    __syncthreads();
    // One fetch-add per touched counter, eight in flight per thread.  The groups of a grid start at
    // different entries (whole waves apart), so that they do not all queue at the same counters.
    constexpr int Q = 8;
    const uint32_t rot = static_cast<uint32_t>(static_cast<uint64_t>(blockIdx.x) * entries / gridDim.x) & ~63u;
    auto entry = [&](uint32_t k) { return k + rot < entries ? k + rot : k + rot - entries; };      // k < entries
    for (uint32_t k0 = threadIdx.x; k0 < entries; k0 += Q * blockDim.x) {
        unsigned long long count[Q];
        int64_t before[Q];
#pragma unroll
        for (int q = 0; q < Q; ++q) {
            const uint32_t k = k0 + q * blockDim.x;
            count[q] = k < entries ? table[entry(k)] : 0ull;
        }
#pragma unroll
        for (int q = 0; q < Q; ++q) {
            if (count[q]) {
                const uint32_t e = entry(k0 + q * blockDim.x);
                before[q] = shm_atomic_fetch_add(c, ctr_off + 8ull * (e % n_ctr), static_cast<int64_t>(count[q]), static_cast<int>(e / n_ctr));
            }
        }
#pragma unroll
        for (int q = 0; q < Q; ++q)
            if (count[q]) table[entry(k0 + q * blockDim.x)] = static_cast<unsigned long long>(before[q]);
    }
    __syncthreads();
    fetch_each([&](uint32_t id) { return static_cast<int64_t>(atomicAdd(table + id, 1ull)); });
    __syncthreads();                                   // the table may be reused once everybody is through
}

// ------------------------------------------------------------------------------------------
// Reverse offload (paper section "Synchronization with Host"): a request to the host proxy is one
// 64-byte message in a ring in pinned host memory.  The sender takes a slot with one atomic
// fetch-and-increment, writes the message with one store instruction (four lanes x 16 bytes, every
// quarter tagged with the slot's generation), and -- if it wants an answer -- polls a completion
// word that it allocated independently of the slot.  The host's consumed count is only read when
// the ring could be full.  shm_offload_send must be called by all 64 lanes of one wave.
// ------------------------------------------------------------------------------------------
#define SHMD_OFFLOAD_SLOTS 4096u
#define SHMD_OFFLOAD_COMPLETIONS 65536u
#define SHMD_OFFLOAD_NONE 0xffffffffu
enum { SHMD_OFFLOAD_NOP = 0, SHMD_OFFLOAD_COPY = 1, SHMD_OFFLOAD_QUIET = 2 };

__device__ __forceinline__ uint64_t shm_wave_first_u64(uint64_t v)
{
    const uint32_t lo = __builtin_amdgcn_readfirstlane(static_cast<uint32_t>(v));
    const uint32_t hi = __builtin_amdgcn_readfirstlane(static_cast<uint32_t>(v >> 32));
    return (static_cast<uint64_t>(hi) << 32) | lo;
}

// Returns the completion ticket, or SHMD_OFFLOAD_NONE if none was asked for.
__device__ __forceinline__ uint64_t shm_offload_send(const shm_dev_ctx &c, uint32_t op, uint32_t me, uint64_t dst, uint64_t src,
                                                     uint64_t n, bool want_completion)
{
    const unsigned lane = __lane_id();
    uint64_t idx = 0, ticket = SHMD_OFFLOAD_NONE;
    uint32_t expired = 0;
    if (lane == 0) {
        idx = __hip_atomic_fetch_add(c.off.head, 1ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if (want_completion) {
            ticket = __hip_atomic_fetch_add(c.off.comp_head, 1ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            if ((ticket & 0xffffffffull) == SHMD_OFFLOAD_NONE)       // the one value that means "none": take the next
                ticket = __hip_atomic_fetch_add(c.off.comp_head, 1ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
        // Flow control, off the critical path: the host's consumed count lives in host memory and
        // reading it crosses the bus, so senders share the largest value any of them has read in a
        // device-memory word and go to the host only when, by that word, the ring could be full.
        if (idx >= SHMD_OFFLOAD_SLOTS &&
            idx - __hip_atomic_load(c.off.consumed_seen, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) >= SHMD_OFFLOAD_SLOTS) {
            const uint64_t t0 = wall_clock64();
            for (;;) {
                const uint64_t seen = __hip_atomic_load(c.off.consumed, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
                __hip_atomic_fetch_max(c.off.consumed_seen, static_cast<unsigned long long>(seen), __ATOMIC_RELAXED,
                                       __HIP_MEMORY_SCOPE_AGENT);
                if (idx - seen < SHMD_OFFLOAD_SLOTS) break;
                if (wall_clock64() - t0 > c.wait_ticks) {
                    __hip_atomic_store(c.status, 1ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
                    expired = 1;
                    break;
                }
                __builtin_amdgcn_s_sleep(8);
            }
        }
    }
    // The host never freed the slot within the wait bound: the request is dropped rather than
    // written over a message the host has not taken (the time-out flag is set; the context's next
    // quiet reports it, and the ring stays stalled at this index).
    if (__builtin_amdgcn_readfirstlane(expired)) return SHMD_OFFLOAD_NONE;
    idx = shm_wave_first_u64(idx);
    ticket = shm_wave_first_u64(ticket);
    const uint32_t tag = static_cast<uint32_t>(idx / SHMD_OFFLOAD_SLOTS) + 1u;
    if (lane < 4) {
        shm_u32x4 q;
        q.w = tag;
        q.z = 0;
        if (lane == 0) {
            q.x = op, q.y = me, q.z = static_cast<uint32_t>(ticket);
        } else {
            const uint64_t v = lane == 1 ? dst : lane == 2 ? src : n;
            q.x = static_cast<uint32_t>(v), q.y = static_cast<uint32_t>(v >> 32);
        }
        shm_u32x4 *slot = reinterpret_cast<shm_u32x4 *>(c.off.ring + (idx & (SHMD_OFFLOAD_SLOTS - 1)) * 16) + lane;
        // system scope: straight to host memory (s_nop: see shm_st16)
        asm volatile("global_store_dwordx4 %0, %1, off sc0 sc1\n\ts_nop 1" ::"v"(slot), "v"(q) : "memory");
    }
    return ticket;
}

// Lane 0 of the calling wave polls the completion word of `ticket` (bounded).
__device__ __forceinline__ void shm_offload_wait(const shm_dev_ctx &c, uint64_t ticket)
{
    if (__lane_id() != 0 || (ticket & 0xffffffffull) == SHMD_OFFLOAD_NONE) return;
    const uint32_t t32 = static_cast<uint32_t>(ticket);
    const uint32_t *word = c.off.completion + (t32 & (SHMD_OFFLOAD_COMPLETIONS - 1));
    const uint32_t want = t32 / SHMD_OFFLOAD_COMPLETIONS + 1u;
    const uint64_t t0 = wall_clock64();
    while (__hip_atomic_load(word, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM) != want) {
        if (wall_clock64() - t0 > c.wait_ticks) {
            __hip_atomic_store(c.status, 1ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
            break;
        }
        __builtin_amdgcn_s_sleep(1);
    }
}

// Work-group put through the host-started copy engine (the paper's leader pattern: group barrier so
// that the source is complete, one wave talks to the host, group barrier).  Blocking: returns when
// the bytes are delivered.  The non-blocking form returns at once; shmx_quiet_offload_wg completes
// everything this PE has offloaded.
__device__ __forceinline__ void shmx_copy_offload_wg(const shm_dev_ctx &c, int me, char *dst, const char *src, size_t n, bool blocking)
{
    __syncthreads();
    if (threadIdx.x < 64 && n != 0) {
        if (threadIdx.x == 0) __builtin_amdgcn_fence(__ATOMIC_RELEASE, "");      // the engine reads memory, not our caches
        const uint64_t ticket = shm_offload_send(c, SHMD_OFFLOAD_COPY, me, reinterpret_cast<uint64_t>(dst),
                                                 reinterpret_cast<uint64_t>(src), n, blocking);
        if (blocking) {
            shm_offload_wait(c, ticket);
            if (threadIdx.x == 0) __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "");  // the engine wrote memory, not our caches
        }
    }
    __syncthreads();
}

__device__ __forceinline__ void shmx_putmem_offload_wg(const shm_dev_ctx &c, int me, uint64_t dst_off, uint64_t src_off, size_t n,
                                                       int pe, bool blocking)
{
    shmx_copy_offload_wg(c, me, shm_ptr(c, dst_off, pe), shm_ptr(c, src_off, me), n, blocking);
}

// The get through the engine: same request with the roles of the two PEs exchanged.  The blocking
// form returns with the bytes readable by every thread of the group; the non-blocking form
// (get_nbi_work_group) leaves them undefined until shmx_quiet_offload_wg.
__device__ __forceinline__ void shmx_getmem_offload_wg(const shm_dev_ctx &c, int me, uint64_t dst_off, uint64_t src_off, size_t n,
                                                       int pe, bool blocking)
{
    shmx_copy_offload_wg(c, me, shm_ptr(c, dst_off, me), shm_ptr(c, src_off, pe), n, blocking);
}

__device__ __forceinline__ void shmx_quiet_offload_wg(const shm_dev_ctx &c, int me)
{
    __syncthreads();
    if (threadIdx.x < 64) {
        const uint64_t ticket = shm_offload_send(c, SHMD_OFFLOAD_QUIET, me, 0, 0, 0, true);
        shm_offload_wait(c, ticket);
        if (threadIdx.x == 0) __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "");
    }
    __syncthreads();
}

// The cutover inside the kernel (paper section "Performance Evaluation"): loads/stores below
// `cutover` bytes, the host-started copy engine from there on.  SHMD_CUTOVER_TUNED asks for the
// threshold measured on MI355X for one work-group of the calling size: it grows with the number of
// work-items, because more lanes move more bytes per microsecond while the engine's start-up time
// (about 14 us through the host) and rate (61 GB/s) stay what they are.
#define SHMD_CUTOVER_TUNED (~static_cast<size_t>(1))
__device__ __forceinline__ size_t shm_tuned_cutover(unsigned work_items)
{
    return work_items <= 1 ? (size_t(16) << 10) : work_items <= 16 ? (size_t(256) << 10) : work_items <= 64 ? (size_t(1) << 20)
                                                                                                             : (size_t(2) << 20);
}
__device__ __forceinline__ size_t shm_resolve_cutover(size_t cutover)
{
    return cutover == SHMD_CUTOVER_TUNED ? shm_tuned_cutover(blockDim.x) : cutover;
}
__device__ __forceinline__ void shmx_putmem_auto_wg(const shm_dev_ctx &c, int me, uint64_t dst_off, uint64_t src_off, size_t n, int pe,
                                                    size_t cutover)
{
    if (c.off.ring != nullptr && n >= shm_resolve_cutover(cutover))
        shmx_putmem_offload_wg(c, me, dst_off, src_off, n, pe, true);
    else
        shmx_putmem_wg(c, me, dst_off, src_off, n, pe);
}
__device__ __forceinline__ void shmx_getmem_auto_wg(const shm_dev_ctx &c, int me, uint64_t dst_off, uint64_t src_off, size_t n, int pe,
                                                    size_t cutover)
{
    if (c.off.ring != nullptr && n >= shm_resolve_cutover(cutover))
        shmx_getmem_offload_wg(c, me, dst_off, src_off, n, pe, true);
    else
        shmx_getmem_wg(c, me, dst_off, src_off, n, pe);
}

// The refinement the paper's implementation notes sketch for the cutover: the engine needs several
// microseconds to start, so the group asks for the engine to move everything past the first
// `cover` bytes, moves those first bytes itself with loads and stores while the engine starts, and
// then waits for both.  is_get exchanges the roles of the PEs.
__device__ __forceinline__ void shmx_rma_covered_wg(const shm_dev_ctx &c, int me, uint64_t dst_off, uint64_t src_off, size_t n, int pe,
                                                    size_t cover, bool is_get)
{
    const size_t head = min(n, (cover + 255) & ~static_cast<size_t>(255));
    const int dpe = is_get ? me : pe, spe = is_get ? pe : me;
    if (c.off.ring != nullptr && n > head)
        shmx_copy_offload_wg(c, me, shm_ptr(c, dst_off + head, dpe), shm_ptr(c, src_off + head, spe), n - head, false);
    else if (n > head)
        return;        // no proxy: the host refuses this mode, nothing is half-done here
    __syncthreads();
    shm_copy_parts<8>(shm_ptr(c, dst_off, dpe), shm_ptr(c, src_off, spe), head, 0, 1);
    __syncthreads();
}

// ------------------------------------------------------------------------------------------
// Strided put/get (paper section "Implementation": blocked and strided RMA use vector copies;
// semantics of OpenSHMEM's iput/iget).  Element i of the source, taken every src_stride elements,
// lands at element i * dst_stride of the destination; elements are 1, 2, 4, 8 or 16 bytes and are
// moved with one load and one store of that width, four elements in flight per thread.  Unit
// strides on both sides are a contiguous block and take the vector copy.
// ------------------------------------------------------------------------------------------
template <typename T>
__device__ __forceinline__ void shm_copy_strided_typed(char *dst, const char *src, size_t dst_stride, size_t src_stride, size_t nelems,
                                                       size_t tid, size_t nthr)
{
    T *d = reinterpret_cast<T *>(dst);
    const T *s = reinterpret_cast<const T *>(src);
    constexpr int U = 4;
    size_t i = tid;
    for (; i + (U - 1) * nthr < nelems; i += U * nthr) {
        T r[U];
#pragma unroll
        for (int u = 0; u < U; ++u) r[u] = s[(i + u * nthr) * src_stride];
#pragma unroll
        for (int u = 0; u < U; ++u) d[(i + u * nthr) * dst_stride] = r[u];
    }
    for (; i < nelems; i += nthr) d[i * dst_stride] = s[i * src_stride];
}

// Elements [first, first + count) of a strided transfer by threads tid of nthr.
__device__ __forceinline__ void shm_copy_strided(char *dst, const char *src, size_t dst_stride, size_t src_stride, size_t first,
                                                 size_t count, uint32_t elem_bytes, size_t tid, size_t nthr)
{
    dst += first * dst_stride * elem_bytes;
    src += first * src_stride * elem_bytes;
    if (dst_stride == 1 && src_stride == 1) {
        shm_copy_coop<4>(dst, src, count * elem_bytes, static_cast<unsigned>(tid), static_cast<unsigned>(nthr));
        return;
    }
    switch (elem_bytes) {
    case 1: shm_copy_strided_typed<uint8_t>(dst, src, dst_stride, src_stride, count, tid, nthr); break;
    case 2: shm_copy_strided_typed<uint16_t>(dst, src, dst_stride, src_stride, count, tid, nthr); break;
    case 4: shm_copy_strided_typed<uint32_t>(dst, src, dst_stride, src_stride, count, tid, nthr); break;
    case 8: shm_copy_strided_typed<uint64_t>(dst, src, dst_stride, src_stride, count, tid, nthr); break;
    default: shm_copy_strided_typed<shm_u32x4>(dst, src, dst_stride, src_stride, count, tid, nthr); break;
    }
}

// Single-thread forms.
__device__ __forceinline__ void shm_iput(const shm_dev_ctx &c, int me, uint64_t dst_off, uint64_t src_off, size_t dst_stride,
                                         size_t src_stride, size_t nelems, uint32_t elem_bytes, int pe)
{
    shm_copy_strided(shm_ptr(c, dst_off, pe), shm_ptr(c, src_off, me), dst_stride, src_stride, 0, nelems, elem_bytes, 0, 1);
}
__device__ __forceinline__ void shm_iget(const shm_dev_ctx &c, int me, uint64_t dst_off, uint64_t src_off, size_t dst_stride,
                                         size_t src_stride, size_t nelems, uint32_t elem_bytes, int pe)
{
    shm_copy_strided(shm_ptr(c, dst_off, me), shm_ptr(c, src_off, pe), dst_stride, src_stride, 0, nelems, elem_bytes, 0, 1);
}

// Work-group forms for `nparts` groups sharing one transfer (this group is `part`): consecutive
// threads take consecutive elements, groups take consecutive blocks of elements.
__device__ __forceinline__ void shmx_iput_parts(const shm_dev_ctx &c, int me, uint64_t dst_off, uint64_t src_off, size_t dst_stride,
                                                size_t src_stride, size_t nelems, uint32_t elem_bytes, int pe, unsigned part,
                                                unsigned nparts)
{
    const size_t per = (nelems + nparts - 1) / nparts;
    const size_t lo = min(nelems, static_cast<size_t>(part) * per), cnt = min(nelems, lo + per) - lo;
    __syncthreads();
    shm_copy_strided(shm_ptr(c, dst_off, pe), shm_ptr(c, src_off, me), dst_stride, src_stride, lo, cnt, elem_bytes, threadIdx.x,
                     blockDim.x);
    __syncthreads();
}
__device__ __forceinline__ void shmx_iget_parts(const shm_dev_ctx &c, int me, uint64_t dst_off, uint64_t src_off, size_t dst_stride,
                                                size_t src_stride, size_t nelems, uint32_t elem_bytes, int pe, unsigned part,
                                                unsigned nparts)
{
    const size_t per = (nelems + nparts - 1) / nparts;
    const size_t lo = min(nelems, static_cast<size_t>(part) * per), cnt = min(nelems, lo + per) - lo;
    __syncthreads();
    shm_copy_strided(shm_ptr(c, dst_off, me), shm_ptr(c, src_off, pe), dst_stride, src_stride, lo, cnt, elem_bytes, threadIdx.x,
                     blockDim.x);
    __syncthreads();
}

// ------------------------------------------------------------------------------------------
// Synchronisation among PEs from inside kernels (paper section "Collective Operations", sync and
// broadcast paragraph): every PE pushes one atomic increment to every other PE's counter -- fire and
// forget, pipelined -- and then waits on its OWN counter for the running total.  Counters only grow;
// the number of syncs a PE has completed is kept next to its counter, so nothing is ever reset.
// One work-group per PE takes part at a time; all of them must be resident together (the team
// launches see to that).  sync orders nothing; barrier = group quiet + sync + acquire.
// ------------------------------------------------------------------------------------------
__device__ __forceinline__ void shmx_sync_all_wg(const shm_dev_ctx &c, int me)
{
    __syncthreads();
    if (threadIdx.x < 64 && c.npes > 1) {
        // lanes 1..npes-1 of the first wave: one increment each, to the other PEs, all in one instruction
        const int j = static_cast<int>(threadIdx.x);
        if (j >= 1 && j < c.npes) {
            int q = me + j;
            if (q >= c.npes) q -= c.npes;
            (void)__hip_atomic_fetch_add(reinterpret_cast<uint64_t *>(shm_ptr(c, c.internal_off + SHMD_INTERNAL_SYNC_COUNT, q)), 1ull,
                                         __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
        if (j == 0) {
            // the number of completed syncs and the first look at the own counter travel together
            uint64_t *epoch = reinterpret_cast<uint64_t *>(shm_ptr(c, c.internal_off + SHMD_INTERNAL_SYNC_EPOCH, me));
            const uint64_t *mine = reinterpret_cast<const uint64_t *>(shm_ptr(c, c.internal_off + SHMD_INTERNAL_SYNC_COUNT, me));
            uint64_t cur = __hip_atomic_load(mine, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            const uint64_t e = __hip_atomic_load(epoch, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) + 1;
            const uint64_t want = e * static_cast<uint64_t>(c.npes - 1);
            const uint64_t t0 = wall_clock64();
            while (cur < want) {
                if (wall_clock64() - t0 > c.wait_ticks) {
                    __hip_atomic_store(c.status, 1ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
                    break;
                }
                __builtin_amdgcn_s_sleep(1);
                cur = __hip_atomic_load(mine, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            }
            __hip_atomic_store(epoch, e, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
    }
    __syncthreads();
}

__device__ __forceinline__ void shmx_barrier_all_wg(const shm_dev_ctx &c, int me)
{
    shmx_quiet_wg();                    // this group's puts are complete and visible ...
    shmx_sync_all_wg(c, me);            // ... before anyone leaves the barrier
    if (threadIdx.x == 0) __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
    __syncthreads();
}

// Broadcast, push form (same paragraph): the root's groups store the block to every PE, inner loop
// over destinations.  Called by the nparts groups of the root only.
__device__ __forceinline__ void shmx_broadcast_push(const shm_dev_ctx &c, int root, uint64_t dst_off, uint64_t src_off, size_t n,
                                                    unsigned part, unsigned nparts)
{
    if (((dst_off | src_off) & 15) == 0) {
        // 16-byte-aligned block: every source vector is loaded once and stored to all PEs (inner loop
        // over destinations, the right-hand neighbour first, the root's own copy last); U loads in
        // flight per thread, consecutive threads on consecutive vectors.
        constexpr int U = 4;
        __syncthreads();
        const char *src = shm_ptr(c, src_off, root);
        const shm_u32x4 *s = reinterpret_cast<const shm_u32x4 *>(src);
        const size_t nvec = n >> 4, gthr = static_cast<size_t>(nparts) * blockDim.x;
        size_t i = static_cast<size_t>(part) * blockDim.x + threadIdx.x;
        for (; i + (U - 1) * gthr < nvec; i += U * gthr) {
            shm_u32x4 r[U];
#pragma unroll
            for (int u = 0; u < U; ++u) r[u] = shm_ld16(s + i + u * gthr);
            for (int j = 0; j < c.npes; ++j) {
                int q = root + 1 + j;
                if (q >= c.npes) q -= c.npes;
                shm_u32x4 *d = reinterpret_cast<shm_u32x4 *>(shm_ptr(c, dst_off, q));
#pragma unroll
                for (int u = 0; u < U; ++u) shm_st16(d + i + u * gthr, r[u]);
            }
        }
        for (; i < nvec; i += gthr) {
            const shm_u32x4 r = shm_ld16(s + i);
            for (int j = 0; j < c.npes; ++j) {
                int q = root + 1 + j;
                if (q >= c.npes) q -= c.npes;
                shm_st16(reinterpret_cast<shm_u32x4 *>(shm_ptr(c, dst_off, q)) + i, r);
            }
        }
        if (part == 0)
            for (size_t b = (nvec << 4) + threadIdx.x; b < n; b += blockDim.x) {       // the last n mod 16 bytes
                const char v = src[b];
                for (int q = 0; q < c.npes; ++q) shm_ptr(c, dst_off, q)[b] = v;
            }
        __syncthreads();
        return;
    }
    if (c.stride == 0 || (c.stride & 15) != 0) {         // partitions that do not share their alignment: a put per destination
        for (int j = 0; j < c.npes; ++j) {
            int q = root + 1 + j;           // the right-hand neighbour first, the root's own copy last
            if (q >= c.npes) q -= c.npes;
            shmx_putmem_parts(c, root, dst_off, src_off, n, q, part, nparts);
        }
        return;
    }
    // Any other addresses: the destinations -- the same offset in equally spaced partitions, so one
    // alignment -- are brought to a 16-byte boundary by a head of single bytes, the source is read ONCE,
    // as aligned words, and every vector is put together and stored to all PEs (a put per destination
    // read the block npes times: 8 PEs, blocks of 40-61 MiB at odd bytes, 19-39 % of the HBM roofline).
    __syncthreads();
    const char *src = shm_ptr(c, src_off, root);
    const unsigned tid = threadIdx.x, nthr = blockDim.x;
    const size_t line = n >= SHM_LINE_HEAD_MIN_BYTES ? SHM_STORE_LINE : 16;      // long blocks: from a boundary of whole lines
    size_t head = (line - (reinterpret_cast<uintptr_t>(shm_ptr(c, dst_off, 0)) & (line - 1))) & (line - 1);
    if (head > n) head = n;
    const size_t body = (n - head) & ~static_cast<size_t>(15), tail = n - head - body;
    auto bytes_to_all = [&](size_t first, size_t count) {
        for (size_t b = first + tid; b < first + count; b += nthr) {
            const char v = src[b];
            for (int q = 0; q < c.npes; ++q) shm_ptr(c, dst_off, q)[b] = v;
        }
    };
    if (part == 0) {
        bytes_to_all(0, head);
        bytes_to_all(head + body, tail);
    }
    if (body) {
        const char *bs = src + head;
        const uint32_t mis = static_cast<uint32_t>(reinterpret_cast<uintptr_t>(bs) & 15), sh = mis & 3;
        const shm_u32x4 *sa = reinterpret_cast<const shm_u32x4 *>(bs - mis);
        const size_t nvec = body >> 4, gthr = static_cast<size_t>(nparts) * nthr;
        auto to_all = [&](size_t i, const shm_u32x4 &r) {
            for (int j = 0; j < c.npes; ++j) {
                int q = root + 1 + j;       // the right-hand neighbour first, the root's own copy last
                if (q >= c.npes) q -= c.npes;
                shm_st16(reinterpret_cast<shm_u32x4 *>(shm_ptr(c, dst_off + head, q)) + i, r);
            }
        };
        // word i + 1 holds at least one byte of the block whenever mis != 0, so it is mapped
        for (size_t i = static_cast<size_t>(part) * nthr + tid; i < nvec; i += gthr) {
            const shm_u32x4 lo = shm_ld16(sa + i);
            if (mis == 0) {
                to_all(i, lo);
                continue;
            }
            const shm_u32x4 hi = shm_ld16(sa + i + 1);
            switch (mis >> 2) {       // uniform over the grid
            case 0: to_all(i, shm_realign<0>(lo, hi, sh)); break;
            case 1: to_all(i, shm_realign<1>(lo, hi, sh)); break;
            case 2: to_all(i, shm_realign<2>(lo, hi, sh)); break;
            default: to_all(i, shm_realign<3>(lo, hi, sh)); break;
            }
        }
    }
    __syncthreads();
}

// ------------------------------------------------------------------------------------------
// Reduction operators (paper section "Collective Operations", reduction paragraph): min, max, sum,
// product, and, or, xor over 8..64-bit integers; min, max, sum, product over float and double.
// Integer sums and products wrap (computed in the unsigned type); min/max keep the earlier operand
// on ties, which also fixes the sign of a zero; the bitwise operators are not defined for the
// floating types (the forms below only keep templates instantiable).
// ------------------------------------------------------------------------------------------
enum { SHMD_OP_MIN = 0, SHMD_OP_MAX = 1, SHMD_OP_SUM = 2, SHMD_OP_PROD = 3, SHMD_OP_AND = 4, SHMD_OP_OR = 5, SHMD_OP_XOR = 6 };

template <typename T> struct shm_arith { typedef T type; };
template <> struct shm_arith<int8_t> { typedef uint8_t type; };
template <> struct shm_arith<int16_t> { typedef uint16_t type; };
template <> struct shm_arith<int32_t> { typedef uint32_t type; };
template <> struct shm_arith<int64_t> { typedef uint64_t type; };

template <typename T> __device__ __forceinline__ T shm_bits_and(T a, T b) { return static_cast<T>(a & b); }
template <typename T> __device__ __forceinline__ T shm_bits_or(T a, T b) { return static_cast<T>(a | b); }
template <typename T> __device__ __forceinline__ T shm_bits_xor(T a, T b) { return static_cast<T>(a ^ b); }
template <> __device__ __forceinline__ float shm_bits_and<float>(float a, float) { return a; }      // never selected for
template <> __device__ __forceinline__ float shm_bits_or<float>(float a, float) { return a; }       // floating types: the
template <> __device__ __forceinline__ float shm_bits_xor<float>(float a, float) { return a; }      // host rejects them
template <> __device__ __forceinline__ double shm_bits_and<double>(double a, double) { return a; }
template <> __device__ __forceinline__ double shm_bits_or<double>(double a, double) { return a; }
template <> __device__ __forceinline__ double shm_bits_xor<double>(double a, double) { return a; }

template <typename T, int OP>
__device__ __forceinline__ T shm_combine(T a, T b)
{
    typedef typename shm_arith<T>::type A;
    if (OP == SHMD_OP_MIN) return b < a ? b : a;
    if (OP == SHMD_OP_MAX) return b > a ? b : a;
    if (OP == SHMD_OP_SUM) return static_cast<T>(static_cast<A>(static_cast<A>(a) + static_cast<A>(b)));
    if (OP == SHMD_OP_PROD) return static_cast<T>(static_cast<A>(static_cast<A>(a) * static_cast<A>(b)));
    if (OP == SHMD_OP_AND) return shm_bits_and<T>(a, b);
    if (OP == SHMD_OP_OR) return shm_bits_or<T>(a, b);
    return shm_bits_xor<T>(a, b);
}

// ------------------------------------------------------------------------------------------
// Collectives callable from inside a kernel (paper section "Proposed Device APIs": broadcast, reduce,
// barrier_all and sync_all have work_group forms).  ONE work-group per PE calls them, all with the
// same arguments, and the groups of all PEs must be resident together: they meet in barriers.
// Each call ends with a barrier, so on return every PE sees the result and may reuse the source.
// ------------------------------------------------------------------------------------------
__device__ __forceinline__ void shmx_broadcast_wg(const shm_dev_ctx &c, int me, uint64_t dst_off, uint64_t src_off, size_t n, int root)
{
    if (me == root) shmx_broadcast_push(c, root, dst_off, src_off, n, 0, 1);
    shmx_barrier_all_wg(c, me);
}

// Every PE's n bytes at src_off land, in PE order, at dst_off of every PE (push: the caller's block
// goes to all PEs, the right-hand neighbour first).
__device__ __forceinline__ void shmx_fcollect_wg(const shm_dev_ctx &c, int me, uint64_t dst_off, uint64_t src_off, size_t n)
{
    for (int j = 0; j < c.npes; ++j) {
        int q = me + 1 + j;
        if (q >= c.npes) q -= c.npes;
        shmx_putmem_wg(c, me, dst_off + static_cast<uint64_t>(me) * n, src_off, n, q);
    }
    shmx_barrier_all_wg(c, me);
}

// dst[i] = src_0[i] OP src_1[i] OP ... in PE order, on every PE (the paper's method: every PE folds
// the whole vector itself from remote loads, so nobody waits for a partial result).  The entry
// barrier makes every PE's source complete and visible; element-aligned offsets; source and
// destination do not overlap.
template <typename T, int OP>
__device__ __forceinline__ void shmx_reduce_wg(const shm_dev_ctx &c, int me, uint64_t dst_off, uint64_t src_off, size_t nelems)
{
    shmx_barrier_all_wg(c, me);
    T *d = reinterpret_cast<T *>(shm_ptr(c, dst_off, me));
    for (size_t i = threadIdx.x; i < nelems; i += blockDim.x) {
        T r = reinterpret_cast<const T *>(shm_ptr(c, src_off, 0))[i];
        for (int p = 1; p < c.npes; ++p) r = shm_combine<T, OP>(r, reinterpret_cast<const T *>(shm_ptr(c, src_off, p))[i]);
        d[i] = r;
    }
    shmx_barrier_all_wg(c, me);
}
