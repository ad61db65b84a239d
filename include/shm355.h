/*
 * shm355 -- device-initiated, work-group-collaborative OpenSHMEM data movement on one MI355X.
 *
 * C ABI of libshm355.so.  Plain pointers and sizes only; no C++ or framework types.
 *
 * Model (paper section "OpenSHMEM Memory and Execution Model"): `npes` processing
 * elements, numbered 0..npes-1, each owning a symmetric heap with identical layout.
 * Here the PEs are logical: PE p's heap is the p-th equal partition of one device
 * allocation, and PE p's work is enqueued on its own HIP stream.  A symmetric
 * address crosses this ABI as a byte offset into the heap and is valid for every
 * PE; the device address is  base[pe] + offset  (paper section "Remote Memory
 * Access": remote = local - local heap base + remote heap base).
 *
 * Because PEs are logical, every call that OpenSHMEM would make "as" a PE names
 * that PE explicitly (`me`).
 *
 * Pointers: `void *heap_base`, `dev_*` arguments are DEVICE pointers; `host`
 * buffers of shm_write/shm_read and all out-parameters (`*out`, `*off`, `*bytes`)
 * are HOST pointers.  Streams are hipStream_t values passed as void*.
 *
 * Errors: every int function returns SHM_OK (0) or a negative code; nothing throws
 * or aborts.  shm_last_error() gives a thread-local text for the last failure.
 *
 * Threads: a context is driven by one host thread at a time (the library takes no locks; the
 * host proxy thread it starts itself shares nothing with the caller but the ring).  Different
 * contexts may be used from different threads.  shm_last_error() is per thread.
 *
 * Work-groups: n_wg is 1 .. 2^20 groups of SHM_WG_SIZE threads unless an entry point
 * states a narrower range.  The team and collective entry points launch n_wg groups
 * for EACH PE as one grid, which must stay below 2^32 threads (n_wg * npes < 2^24).
 *
 * Completion: shm_launch_* and shm_putmem/shm_getmem are asynchronous on the
 * stream of the calling PE (team launches: on the team stream, PE 0's).  They are
 * complete, and their effects visible to every PE and to shm_read, after
 * shm_quiet(me) (that PE's work) or shm_barrier_all (everyone's).  A bounded device
 * wait that expired is reported by the next shm_quiet/shm_barrier_all as
 * SHM_ETIMEOUT.
 */
#ifndef SHM355_H
#define SHM355_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define SHM_MAX_PES        32          /* most logical PEs in one context */
#define SHM_WG_SIZE        256         /* threads per work-group of every launch */
#define SHM_INTERNAL_BYTES 65536       /* tail of each partition kept for the library (arrival counters) */
#define SHM_NULL_OFF       UINT64_MAX  /* offset returned by a zero-byte allocation */

enum { SHM_OK = 0, SHM_EINVAL = -1, SHM_EPE = -2, SHM_ERANGE = -3, SHM_ENOMEM = -4,
       SHM_EHIP = -5, SHM_ETIMEOUT = -6, SHM_ENODEV = -7 };

enum { SHM_PATH_AUTO = 0, SHM_PATH_LDST = 1, SHM_PATH_SDMA = 2, SHM_PATH_MEMCPY = 3 };
enum { SHM_SIGNAL_SET = 0, SHM_SIGNAL_ADD = 1 };
enum { SHM_CMP_EQ = 0, SHM_CMP_NE = 1, SHM_CMP_GT = 2, SHM_CMP_GE = 3, SHM_CMP_LT = 4, SHM_CMP_LE = 5 };
enum { SHM_INIT_DEFAULT = 0, SHM_INIT_NO_DEVICE = 1 };
enum { SHM_AMO_FETCH = 0, SHM_AMO_SET = 1, SHM_AMO_SWAP = 2, SHM_AMO_COMPARE_SWAP = 3,
       SHM_AMO_FETCH_ADD = 4, SHM_AMO_ADD = 5, SHM_AMO_FETCH_INC = 6, SHM_AMO_INC = 7 };
enum { SHM_STORM_FETCH_ADD = 0, SHM_STORM_ADD = 1, SHM_STORM_CSWAP_LOOP = 2, SHM_STORM_PLAIN_STORE = 3, SHM_STORM_FETCH_ADD_WG = 4 };
enum { SHM_REDUCE_DUPLICATE = 0, SHM_REDUCE_SPLIT = 1 };
enum { SHM_COLL_FCOLLECT = 0, SHM_COLL_BROADCAST = 1 };
enum { SHM_TEAM_SYNC_OFF = 0, SHM_TEAM_SYNC_FULL = 1, SHM_TEAM_SYNC_TRACKED = 2 };
enum { SHM_OP_MIN = 0, SHM_OP_MAX = 1, SHM_OP_SUM = 2, SHM_OP_PROD = 3, SHM_OP_AND = 4, SHM_OP_OR = 5, SHM_OP_XOR = 6 };
enum { SHM_INT8 = 0, SHM_UINT8 = 1, SHM_INT16 = 2, SHM_UINT16 = 3, SHM_INT32 = 4, SHM_UINT32 = 5, SHM_INT64 = 6, SHM_UINT64 = 7,
       SHM_FLOAT32 = 8, SHM_FLOAT64 = 9 };

typedef struct shm_ctx shm_ctx;

/* ---- set-up (host only; paper section "Proposed Device APIs": initialisation, finalisation and
 *      memory management are host-only) ------------------------------------------------------- */

/* Create a context of `npes` PEs (1..SHM_MAX_PES) with `heap_bytes` per PE (multiple of 4096,
 * larger than SHM_INTERNAL_BYTES).  heap_base: device pointer to npes*heap_bytes bytes, 256-byte
 * aligned, borrowed (caller frees after shm_finalize); NULL = the library allocates and owns it.
 * streams: npes hipStream_t values, borrowed; NULL = the library creates non-blocking streams.
 * The internal tail of every partition is zeroed.  *out receives the context. */
int shm_init(int npes, size_t heap_bytes, void *heap_base, void *const *streams, shm_ctx **out);

/* As shm_init with flags.  SHM_INIT_NO_DEVICE builds a context that makes no HIP call at all
 * (heap_base may be any non-NULL value, streams are ignored): allocation, argument checking and
 * the cutover policy work; everything that would touch the device returns SHM_ENODEV after its
 * arguments have been validated. */
int shm_init_ex(int npes, size_t heap_bytes, void *heap_base, void *const *streams, unsigned flags, shm_ctx **out);

/* Waits for all streams, releases what the library owns.  The context is invalid afterwards. */
int shm_finalize(shm_ctx *ctx);

int         shm_n_pes(const shm_ctx *ctx);           /* npes, or SHM_EINVAL */
size_t      shm_heap_bytes(const shm_ctx *ctx);      /* bytes a caller can allocate per PE (partition minus internal tail) */
const char *shm_last_error(void);                    /* text of this thread's last error; never NULL */

/* Symmetric allocation (collective by construction: one offset for all PEs).  align: power of
 * two, 0 = 256.  bytes == 0 succeeds with *off = SHM_NULL_OFF.  SHM_ENOMEM when no gap fits.
 * shm_calloc also zeroes the block on every PE (synchronous).  shm_free(SHM_NULL_OFF) is a no-op;
 * an offset that is not a live block is SHM_EINVAL. */
int shm_malloc(shm_ctx *ctx, size_t bytes, size_t align, uint64_t *off);
int shm_calloc(shm_ctx *ctx, size_t bytes, size_t align, uint64_t *off);
int shm_free(shm_ctx *ctx, uint64_t off);

/* Device address of symmetric offset `off` on PE `pe` (paper section "Remote Memory Access",
 * address rule); NULL on a bad PE or an offset outside the partition. */
void *shm_ptr(const shm_ctx *ctx, uint64_t off, int pe);

/* Test staging, not OpenSHMEM: synchronous copies between a host buffer and PE `pe`'s heap. */
int shm_write(shm_ctx *ctx, int pe, uint64_t off, const void *host, size_t n);
int shm_read(shm_ctx *ctx, int pe, uint64_t off, void *host, size_t n);

/* ---- host-initiated RMA and ordering (paper section "Architectural Overview": host-initiated
 *      routines mirror the device ones; section "Xe-Link Capabilities": copy engines for large and
 *      non-blocking transfers) ----------------------------------------------------------------- */

/* PE `me` copies n bytes from its offset src_off to offset dst_off of PE `pe` (put), or from PE
 * `pe`'s src_off to its own dst_off (get), with hipMemcpyAsync in order on me's stream.
 * Overlapping ranges on one PE are SHM_EINVAL. */
int shm_putmem(shm_ctx *ctx, int me, uint64_t dst_off, uint64_t src_off, size_t n, int pe);
int shm_getmem(shm_ctx *ctx, int me, uint64_t dst_off, uint64_t src_off, size_t n, int pe);

/* quiet: all of PE me's outstanding operations are complete and visible (host wait on its stream,
 * on its copy-engine transfers, and -- while the host proxy runs -- on the engine transfers its
 * kernels started through the ring without waiting for them: the PE-wide quiet that completes a
 * kernel's put_nbi / get_nbi).  fence: orders me's earlier operations before its later ones;
 * the stream is in-order, so only host-started engine transfers need waiting for.  barrier_all:
 * quiet for every PE.  All three report an expired device wait (SHM_ETIMEOUT); quiet and
 * barrier_all also report an engine transfer a kernel asked for and the proxy could not start
 * (SHM_EHIP). */
int shm_quiet(shm_ctx *ctx, int me);
int shm_fence(shm_ctx *ctx, int me);
int shm_barrier_all(shm_ctx *ctx);

/* ---- policy (paper section "Performance Evaluation": the cutover between stores from kernel
 *      threads and the copy engine depends on message size and on the number of active work-items) */

/* Transfer paths.  LDST: loads/stores from kernel threads.  SDMA: the GPU's copy engines (driven
 * through the HSA runtime; the host first waits for the calling PE's stream, the transfer then runs
 * asynchronously, like a non-blocking put, until that PE's quiet/fence/barrier or next launch).
 * MEMCPY: hipMemcpyAsync in stream order -- on one device the runtime executes it as a copy kernel
 * of its own, not on an engine; kept as a reference curve.
 * With SHM_PATH_AUTO a transfer of n bytes by n_wg work-groups uses SDMA iff
 * n >= cutover(class of n_wg); classes are n_wg <= 1, <= 4, <= 64, > 64.  SIZE_MAX = never.
 * Defaults are the thresholds measured on MI355X with 8 PEs transferring at once (the paper sets its
 * own the same way, internally), and they depend on whether every PE's stream has a hardware queue of
 * its own: the HIP runtime creates GPU_MAX_HW_QUEUES queues per process (4 unless the environment
 * says otherwise), and with fewer queues than PEs the put kernels of different PEs take turns, which
 * halves what loads/stores deliver while the engines are not affected.  shm_init reads that variable:
 *   queues >= npes: 512 KiB for one group per PE, never for more;
 *   queues <  npes: 256 KiB for one group per PE, 2 MiB for up to four, never for more.
 * A context whose copy engines are unavailable keeps AUTO on loads/stores. */
int shm_set_cutover(shm_ctx *ctx, int n_wg, size_t bytes);
int shm_get_cutover(const shm_ctx *ctx, int n_wg, size_t *bytes);
/* Which path AUTO would take: writes SHM_PATH_LDST or SHM_PATH_SDMA to *path. */
int shm_choose_path(const shm_ctx *ctx, size_t n, int n_wg, int *path);

/* The cutover of the collectives (paper section "Performance Evaluation", the fcollect and broadcast
 * experiments: the threshold of a collective also depends on the number of PEs and is tuned per
 * collective).  `collective` is SHM_COLL_FCOLLECT or SHM_COLL_BROADCAST; classes of n_wg as above;
 * bytes are per PE.  With SHM_PATH_AUTO a collective of bytes_per_pe >= the threshold is done by
 * host-started copies -- SHM_PATH_MEMCPY, which on one device outruns the engines for these
 * many-copy patterns -- and by the push kernel below it.  Defaults measured on MI355X:
 * fcollect 512 KiB / 2 MiB / never / never up to 4 PEs and 2 MiB / 8 MiB / never / never beyond
 * (n_wg <= 1, <= 4, <= 64, more); broadcast 256 KiB / 1 MiB / 16 MiB / never for any number of PEs. */
int shm_set_collective_cutover(shm_ctx *ctx, int collective, int n_wg, size_t bytes);
int shm_get_collective_cutover(const shm_ctx *ctx, int collective, int n_wg, size_t *bytes);
/* Which path AUTO would take for that collective: SHM_PATH_LDST or SHM_PATH_MEMCPY. */
int shm_choose_collective_path(const shm_ctx *ctx, int collective, size_t bytes_per_pe, int n_wg, int *path);

/* Upper bound for every device-side wait, in microseconds (default 2 000 000; must be > 0). */
int shm_set_wait_timeout_us(shm_ctx *ctx, uint64_t us);
/* Team launches run on PE 0's stream.  SHM_TEAM_SYNC_FULL (default): they first wait for all PE
 * streams and all PE streams then wait for them: whatever was enqueued before a team launch, on any
 * PE's stream, is ordered before it, and whatever is enqueued after it is ordered behind it.  That
 * holds for a team launch with nothing to move (zero bytes or elements) too, and on the copy-engine
 * path, where the call then returns only after the engines have finished (they are not on the
 * streams, so only the host can order other PEs' later work behind them).
 * SHM_TEAM_SYNC_TRACKED gives the same ordering for everything enqueued THROUGH THIS LIBRARY at a
 * fraction of the cost (a full join and fork of 8 streams costs about 80 us of host time per team
 * launch): a team launch waits only for the PE streams the library has used since the last one,
 * and a PE stream catches up with the team stream when the library next uses it (or in shm_quiet).
 * Work the caller enqueues on a PE stream by other means (a kernel of its own on shm_stream(pe),
 * a stream the context borrowed) is not seen by the tracking: order it yourself or use FULL.
 * SHM_TEAM_SYNC_OFF: the caller orders streams itself, engine transfers stay asynchronous until a
 * quiet, and an empty team launch does nothing but wait for engine transfers in flight. */
int shm_set_team_sync(shm_ctx *ctx, int mode);

/* ---- kernels of the caller's own (paper section "Proposed Device APIs": the operations are called
 *      from inside application kernels) --------------------------------------------------------- */

/* The device functions of csrc/shm_device.hpp take a small by-value view of the context, a
 * `shm_dev_ctx`, as their first argument.  shm_device_context copies that view to the HOST buffer
 * `out`; out_bytes must equal shm_device_context_bytes() (= sizeof(shm_dev_ctx) of the library's
 * build, so a kernel built against another layout is refused instead of misread).  Pass the view to
 * a kernel by value.  It names the heap partitions, the number of PEs, the bound of device-side
 * waits in force and, while the host proxy runs, the reverse-offload ring: take a new one after
 * shm_set_wait_timeout_us, shm_proxy_start or shm_proxy_stop.  shm_stream gives PE `pe`'s stream
 * (a hipStream_t; NULL on error or for a context without a device), so that such kernels can be
 * ordered with the library's own launches; a kernel on any other stream is the caller's to order.
 * What such a kernel has put is complete after shm_quiet of the PE whose stream it ran on. */
size_t shm_device_context_bytes(void);
int    shm_device_context(const shm_ctx *ctx, void *out, size_t out_bytes);
void  *shm_stream(const shm_ctx *ctx, int pe);
/* Announces that the caller is about to enqueue work of its own on PE `pe`'s stream.  Needed under
 * SHM_TEAM_SYNC_TRACKED only (harmless otherwise): PE pe's engine transfers are finished, its
 * stream catches up with the team stream, and the next team launch waits for that stream. */
int    shm_stream_used(shm_ctx *ctx, int pe);

/* ---- kernel-launch entry points that exercise the device API ---------------------------------- */

/* Work-group put/get (paper section "Proposed Device APIs", the work_group extensions; section
 * "Remote Memory Access": multi-threaded vectorised copy).  n_wg work-groups of SHM_WG_SIZE
 * threads share the message; which bytes a group moves is not observable and is chosen for the
 * memory system (see shm_device.hpp) -- including how many of the n_wg groups take part: a launch may
 * run fewer groups than it was asked for (long messages, short messages dealt to very many groups,
 * long collectives), never more.  path: LDST = kernel on me's stream, SDMA = copy engine,
 * MEMCPY = runtime copy on me's stream, AUTO = LDST or SDMA by cutover.  Any byte alignment; n may
 * be 0.  A message of 32 MiB or more asked of 32-100 groups, and one of 128 MiB or more asked of a
 * group per compute unit or more, is moved in pieces drawn from counter
 * pairs in PE me's part of the library's tail of the heap (it sets itself back): me's launches follow
 * one another on its stream; a caller who replays recorded ones elsewhere keeps them from overlapping. */
int shm_launch_wg_put(shm_ctx *ctx, int me, int pe, uint64_t dst_off, uint64_t src_off, size_t n, int n_wg, int path);
int shm_launch_wg_get(shm_ctx *ctx, int me, int pe, uint64_t dst_off, uint64_t src_off, size_t n, int n_wg, int path);

/* Team form: every PE p does the same put/get towards PE (p + pe_shift) mod npes, each with n_wg
 * work-groups, as ONE grid of npes*n_wg groups on the team stream (LDST) or as npes copies, one
 * per PE, on the engines (SDMA) or the PEs' own streams (MEMCPY).  Long LDST messages (32 MiB or
 * more per PE asked of about 128 groups or more, from 128 MiB also of fewer; two PEs or more; any
 * byte addresses) are moved by at most about 128 groups per PE (a whole number of groups per compute
 * unit in all, never more than asked for) that stay in the kernel
 * and draw 32 KiB pieces, counted from the destination's next 1 KiB boundary, from counters in the library's tail of the heap; the counters set themselves
 * back, so such a launch can be recorded into a HIP graph and replayed like any other.  The library's
 * own launches follow one another on the team stream; a caller who replays recorded team launches of
 * one context on streams of their own keeps them from overlapping, as they share those counters
 * (long fcollects, collects, broadcasts and split reductions share a second pair in the same way). */
int shm_launch_wg_put_all(shm_ctx *ctx, int pe_shift, uint64_t dst_off, uint64_t src_off, size_t n, int n_wg, int path);
int shm_launch_wg_get_all(shm_ctx *ctx, int pe_shift, uint64_t dst_off, uint64_t src_off, size_t n, int n_wg, int path);

/* Measurement aid for the paper's put experiment (section "Performance Evaluation": bandwidth and
 * latency of the work-group put as issued from a running kernel): one kernel of n_wg groups on
 * me's stream performs the same put `reps` times, each followed by the group's quiet, and reads
 * the device wall clock before and after.  dev_ticks (device pointer to two uint64, initialised by
 * the caller to UINT64_MAX and 0) receives the earliest start and the latest end over the groups that
 * have a share of the message (a group without one returns from every put at once; when it is started is
 * launch overhead),
 * combined with atomic min/max so that several launches can share one pair.  shm_wall_clock_khz
 * gives the tick rate. */
int shm_launch_wg_put_timed(shm_ctx *ctx, int me, int pe, uint64_t dst_off, uint64_t src_off, size_t n, int n_wg, int reps,
                            uint64_t *dev_ticks);
int shm_wall_clock_khz(const shm_ctx *ctx);

/* Measurement aid: the one-direction ceilings of the memory system, taken with the access forms
 * and the launch shape of the long-message team put (paper section "Performance Evaluation" reports
 * bandwidth against what the link can carry; here the "link" is HBM, whose read, write and copy
 * rates differ).  One grid of npes*n_wg groups on the team stream; every PE p handles n bytes
 * (a multiple of 65536; offsets 16-byte aligned, inside the heap):
 *   SHM_PROBE_READ   p only reads [src_off, src_off+n) of its own partition;
 *   SHM_PROBE_WRITE  p only writes a pattern to [dst_off, dst_off+n) of PE (p+1) mod npes;
 *   SHM_PROBE_COPY   the team put itself (shm_launch_wg_put_all with shift 1, loads/stores);
 *   SHM_PROBE_READ_FRONT, SHM_PROBE_WRITE_FRONT   as READ / WRITE, but the n_wg groups of a PE sweep
 *                    its block together, 4 KiB per group and step (no tiles): the order in which this
 *                    chip writes fastest with fixed shares;
 *   SHM_PROBE_READ_TICKETS, SHM_PROBE_WRITE_TICKETS   as READ / WRITE with the walk of the long put
 *                    itself: the n_wg groups of a PE (128 is what the put runs) draw 32 KiB pieces of
 *                    its block by ticket.  The best form of a direction is that direction's ceiling.
 * READ leaves memory unchanged; WRITE overwrites the destination with a pattern of no meaning. */
enum { SHM_PROBE_READ = 0, SHM_PROBE_WRITE = 1, SHM_PROBE_COPY = 2, SHM_PROBE_READ_FRONT = 3, SHM_PROBE_WRITE_FRONT = 4,
       SHM_PROBE_READ_TICKETS = 5, SHM_PROBE_WRITE_TICKETS = 6 };
int shm_launch_stream_probe(shm_ctx *ctx, int kind, uint64_t dst_off, uint64_t src_off, size_t n, int n_wg);

/* ---- device-initiated copy-engine transfers (paper section "Synchronization with Host": the
 *      reverse-offload ring; section "Performance Evaluation": the cutover taken inside the kernel) */

/* Start / stop the host proxy thread and its ring (64-byte messages in pinned host memory).  While
 * it runs, kernels can ask the host to start an SDMA transfer.  Start waits for all streams and
 * resets the ring; stop waits for all streams, lets the thread take what is still in the ring and
 * finish the transfers it started, then joins it.  shm_finalize stops it too.
 * shm_proxy_stats reports how many requests and how many engine copies the proxy has served since
 * its start (either pointer may be NULL). */
int shm_proxy_start(shm_ctx *ctx);
int shm_proxy_stop(shm_ctx *ctx);
int shm_proxy_stats(const shm_ctx *ctx, uint64_t *requests, uint64_t *copies);

/* One kernel of n_wg groups (1..1024) of wg_size threads (1..1024: the paper varies the work-items
 * per work-group; modes 1-3 talk to the host with one whole wave and need a multiple of 64) on me's
 * stream puts n bytes from me's src_off to pe's dst_off `reps` times; group g owns the g-th
 * contiguous 256-byte-aligned share.  mode 0: loads/stores and group quiet; 1: reverse offload to
 * a copy engine, blocking; 2: cutover inside the kernel (share size >= cutover bytes -> engine,
 * else loads/stores); 3: non-blocking offload followed by an offload quiet.  Modes 1-3 need the proxy.  dev_ticks as for shm_launch_wg_put_timed. */
int shm_launch_put_device_initiated(shm_ctx *ctx, int me, int pe, uint64_t dst_off, uint64_t src_off, size_t n, int n_wg, int wg_size,
                                    int mode, size_t cutover, int reps, uint64_t *dev_ticks);

/* The general form: put (is_get 0) or get (is_get 1; n bytes from pe's src_off to me's dst_off:
 * the paper's get_work_group and get_nbi_work_group, section "Proposed Device APIs").  Modes 0-3 as
 * above (a get by loads/stores needs no quiet); mode 4 is the refinement the paper's implementation
 * notes sketch for the cutover: the engine moves all but the first `cover` bytes of a group's share
 * while the group moves those first bytes with loads and stores, covering the engine's start-up
 * time; then both are waited for; mode 5 is put_nbi / get_nbi with no quiet inside the kernel:
 * the transfer is complete after shm_quiet(me) or shm_barrier_all (no consume_off then).
 * consume_off (get only; SHM_NO_CONSUME = none): offset on PE me of n bytes that do not overlap the
 * transfer; the group copies its share of the destination there
 * before the first get and after every get, from inside the kernel, so the buffer shows what the
 * kernel itself reads after a get.  dev_ticks may be NULL. */
#define SHM_NO_CONSUME UINT64_MAX
/* As `cutover` of mode 2: the threshold measured on MI355X for one work-group of wg_size work-items
 * (16 KiB for 1, 256 KiB up to 16, 1 MiB up to 64, 2 MiB beyond). */
#define SHM_CUTOVER_TUNED (SIZE_MAX - 1)
int shm_launch_rma_device_initiated(shm_ctx *ctx, int me, int pe, uint64_t dst_off, uint64_t src_off, size_t n, int n_wg, int wg_size,
                                    int is_get, int mode, size_t cutover, size_t cover, uint64_t consume_off, int reps,
                                    uint64_t *dev_ticks);

/* Scalar put and get (paper section "Remote Memory Access": the ishmem_long_p example -- address
 * translation, then one store; g is the matching load).  n_wg groups of 256 work-items on me's
 * stream; work-item i handles elements i, i + 256 n_wg, ...  is_get 0: element i of me's src_off is
 * p'ed to pe's dst_off.  is_get 1: element i of pe's src_off is g'ed and stored to me's dst_off.
 * elem_bytes in {1, 2, 4, 8}; offsets element-aligned.  Delivered after shm_quiet(me). */
int shm_launch_scalar_pg(shm_ctx *ctx, int me, int pe, uint64_t dst_off, uint64_t src_off, size_t nelems, int elem_bytes, int is_get,
                         int n_wg);

/* The sub-group forms (paper section "Proposed Device APIs": sub-group extensions; a sub-group is a
 * 64-lane wave here) in one kernel on me's stream.  Wave w of n_waves (1..4096) owns the w-th
 * 16-byte-rounded share of the n-byte message.  Producer waves (PE me): wave put of the share from
 * src_off to pe's dst_off, fence, then pe's flag word flag_off + 8w := 1.  Consumer waves (PE pe):
 * wait until that flag == 1 (bounded), store the value signal_fetch returns to out_off + 8w, then
 * wave-get the share from pe's own dst_off into back_off.  The caller zeroes the flags first.
 * All buffers on pe are pairwise disjoint (SHM_EINVAL otherwise); the grid must fit the device as a
 * whole (SHM_EINVAL). */
int shm_launch_wave_exchange(shm_ctx *ctx, int me, int pe, uint64_t dst_off, uint64_t src_off, uint64_t back_off, size_t n, int n_waves,
                             uint64_t flag_off, uint64_t out_off);

/* Single-thread put/get (paper section "Performance Evaluation", first experiment: ishmem_put and
 * ishmem_get called by one work-item): one thread of one kernel on me's stream moves n bytes `reps`
 * times, a quiet after each put.  dev_ticks as above, or NULL. */
int shm_launch_thread_rma(shm_ctx *ctx, int me, int pe, uint64_t dst_off, uint64_t src_off, size_t n, int is_get, int reps,
                          uint64_t *dev_ticks);

/* Strided put/get (paper section "Implementation": blocked and strided RMA on vector copies;
 * OpenSHMEM iput/iget).  iput: element i of me's source, i = 0..nelems-1, taken every src_stride
 * elements from src_off, becomes the element at dst_off + i * dst_stride elements on pe; bytes
 * between destination elements are untouched.  iget: the source is on pe, the destination on me.
 * elem_bytes in {1, 2, 4, 8, 16}; strides >= 1, in elements; offsets multiples of elem_bytes.
 * n_wg = 0: one work-item does it all (the single-thread call); n_wg >= 1: that many work-groups
 * share the elements (the work-group call).  Delivered after shm_quiet(me).  SHM_EINVAL for a bad
 * element size, stride, alignment or overlap on one PE; SHM_ERANGE if either side leaves the heap. */
int shm_launch_iput(shm_ctx *ctx, int me, int pe, uint64_t dst_off, uint64_t src_off, int64_t dst_stride, int64_t src_stride,
                    size_t nelems, int elem_bytes, int n_wg);
int shm_launch_iget(shm_ctx *ctx, int me, int pe, uint64_t dst_off, uint64_t src_off, int64_t dst_stride, int64_t src_stride,
                    size_t nelems, int elem_bytes, int n_wg);

/* Ring micro-benchmark: the leader wave of each of n_wg groups (1..4096) sends `reps` empty
 * requests; blocking != 0: it waits for every answer (round trips), else it fires them and waits
 * once at the end (request rate).  dev_ticks as above. */
int shm_launch_offload_nop(shm_ctx *ctx, int me, int n_wg, int reps, int blocking, uint64_t *dev_ticks);

/* Put with signal (OpenSHMEM 1.5 semantics, which the paper's feature list adopts): after all n
 * bytes are visible on PE `pe`, its 64-bit word at sig_off (8-byte aligned) is set to sig_val
 * (SET) or increased by it modulo 2^64 (ADD), exactly once however many groups shared the copy.
 * n == 0 still signals.  Always the kernel path. */
int shm_launch_wg_put_signal(shm_ctx *ctx, int me, int pe, uint64_t dst_off, uint64_t src_off, size_t n,
                             uint64_t sig_off, uint64_t sig_val, int sig_op, int n_wg);

/* One work-group of PE `me` waits until  cmp(word at sig_off on me, val)  holds (unsigned), with
 * acquire semantics, and stores the satisfying value to *dev_out (device pointer, may be NULL).
 * The wait is bounded by the wait timeout. */
int shm_launch_signal_wait_until(shm_ctx *ctx, int me, uint64_t sig_off, int cmp, uint64_t val, uint64_t *dev_out);

/* Point-to-point synchronisation on 64-bit SIGNED variables of PE me's own heap (paper section
 * "Proposed Device APIs": callable from the device; semantics of OpenSHMEM 1.5 wait_until, test and
 * their all / any / some forms).  One thread of PE me looks at the nelems int64 variables at
 * ivars_off (8-byte aligned; the single forms use the first).  dev_status (device pointer or NULL):
 * nelems ints, nonzero = that variable is not part of the set.  kind: SHM_SYNC_WAIT, _WAIT_ALL,
 * _WAIT_ANY, _WAIT_SOME block (bounded by the wait timeout) until the variable / every selected
 * variable / at least one satisfies cmp(variable, val); SHM_SYNC_TEST, _TEST_ALL, _TEST_ANY,
 * _TEST_SOME look once.  dev_out (device pointer, 1 + nelems uint64): [0] = the satisfying value
 * (WAIT), 1 or 0 (WAIT_ALL, TEST, TEST_ALL), the index of a satisfying variable or UINT64_MAX
 * (the ANY forms), the number of satisfying variables (the SOME forms), whose indices follow in
 * [1 ..].  An empty set: ALL is satisfied, ANY gives UINT64_MAX, SOME gives 0, without waiting. */
enum { SHM_SYNC_WAIT = 0, SHM_SYNC_WAIT_ALL = 1, SHM_SYNC_WAIT_ANY = 2, SHM_SYNC_WAIT_SOME = 3,
       SHM_SYNC_TEST = 4, SHM_SYNC_TEST_ALL = 5, SHM_SYNC_TEST_ANY = 6, SHM_SYNC_TEST_SOME = 7 };
int shm_launch_sync_set(shm_ctx *ctx, int me, uint64_t ivars_off, size_t nelems, const int *dev_status, int kind, int cmp, int64_t val,
                        uint64_t *dev_out);

/* One work-item of PE `me` performs one 64-bit atomic `op` (SHM_AMO_*) on offset `off` (8-byte
 * aligned) of PE `pe` (paper section "Xe-Link Capabilities": atomics from GPU threads; section
 * "Proposed Device APIs": AMOs are scalar).  *dev_out (device pointer or NULL) receives the
 * fetched value for the fetching ops. */
int shm_launch_amo(shm_ctx *ctx, int me, int pe, uint64_t off, int op, int64_t operand, int64_t cond, int64_t *dev_out);

/* Benchmark configuration 1.  PE 0, one work-group: work-group put of n bytes from data_off to
 * data_off on PE 1; quiet; zero-byte put-with-signal SET 1 on flag_off.  PE 1, one work-group on
 * its own stream: wait flag == 1, then work-group get of PE 0's n bytes at data_off into its
 * back_off.  Needs npes >= 2. */
int shm_launch_pingflag(shm_ctx *ctx, uint64_t data_off, uint64_t back_off, size_t n, uint64_t flag_off);

/* Benchmark configuration 3, one grid on the team stream.  Every PE p sends n_chunks chunks
 * (chunk k = chunk_bytes at src_off + k*chunk_bytes) to slot k (slot_off + k*chunk_bytes) of PE
 * (p+1) mod npes with put-with-signal ADD 1, using n_wg_prod producer groups; n_wg_cons consumer
 * groups of every PE wait for chunk k (signal >= k+1) and add it, read as bf16 and widened
 * exactly, into a float32 accumulator kept in registers, in chunk order; at the end the
 * accumulator is stored at acc_off (chunk_bytes/2 floats).
 *   n_sig == 1: one signal word at sig_off; the producer groups share every chunk, count their
 *     arrivals, and the last one signals.
 *   n_sig == n_wg_prod == n_wg_cons: lanes.  Producer group j puts the j-th share of every chunk
 *     with its own put-with-signal on word sig_off + 8*j; consumer group j waits on that word and
 *     accumulates that share.
 * chunk_bytes must be a multiple of 16 and all offsets 16-byte aligned; the n_sig signal words
 * must be zero on entry (each ends at n_chunks); the grid must fit on the GPU at once (else
 * SHM_EINVAL). */
int shm_launch_ring_pipeline(shm_ctx *ctx, uint64_t src_off, uint64_t slot_off, uint64_t sig_off, uint64_t acc_off,
                             size_t chunk_bytes, int n_chunks, int n_wg_prod, int n_wg_cons, int n_sig);

/* The same ring for callers that cannot allocate device memory or have the library do so on their
 * behalf: code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  It
 * allocates nothing and calls no allocating routine: the arrival counters of the chunks, which
 * shm_launch_ring_pipeline keeps in the heap's library-owned tail, are taken from a static device
 * array inside the library (32 PEs x SHM_STATIC_RING_MAX_CHUNKS counters of 8 bytes = 256 KiB,
 * held by every GPU the library runs on until the process ends) and cleared by a small kernel
 * before the ring starts.  n_chunks above SHM_STATIC_RING_MAX_CHUNKS is refused with SHM_EINVAL;
 * everything else -- arguments, results, completion, errors -- is as for shm_launch_ring_pipeline.
 * All calls on one GPU share the one array: two such calls that overlap in time on a GPU (from two
 * contexts, or from streams the caller has not ordered) race on the counters and must be
 * serialised by the caller. */
#define SHM_STATIC_RING_MAX_CHUNKS 1024
int shm_launch_ring_pipeline_static(shm_ctx *ctx, uint64_t src_off, uint64_t slot_off, uint64_t sig_off, uint64_t acc_off,
                                    size_t chunk_bytes, int n_chunks, int n_wg_prod, int n_wg_cons, int n_sig);

/* Benchmark configuration 4, one grid on the team stream.  Work-item g < n_items performs
 * ops_per_item atomics; its j-th target is dev_targets[g*ops_per_item + j] = pe*n_ctr + index,
 * i.e. the int64 counter at ctr_off + 8*index on that PE.  kind: FETCH_ADD(+1) | ADD(+1, no
 * return) | CSWAP_LOOP (increment built from compare-swap) | PLAIN_STORE (not atomic; a timing
 * ceiling only) | FETCH_ADD_WG (the same fetch-adds batched by work-groups of 1024 work-items,
 * at most one group per compute unit: a group counts its increments per counter in LDS, sends
 * one fetch-add per counter it touched and hands every increment its own fetched value; an
 * extension -- the paper, section "Proposed Device APIs", gives the atomics no group form --
 * with the same observable result, i.e. the fetched values of a counter are those of one valid
 * order of its increments; needs n_ctr * npes <= 16384, SHM_EINVAL otherwise).  dev_fetched (or
 * NULL): [n_items*ops_per_item] fetched values.  dev_checksum (or NULL): one uint64 per 256
 * consecutive work-items, the sum of what they fetched.  n_items is 1 .. 2^32 - 256 (one grid);
 * n_ctr * npes <= 65536; ops_per_item 1 .. 4096; dev_targets 16-byte aligned. */
int shm_launch_amo_storm(shm_ctx *ctx, uint64_t ctr_off, int n_ctr, const uint16_t *dev_targets, uint64_t n_items,
                         int ops_per_item, int kind, int64_t *dev_fetched, uint64_t *dev_checksum);

/* Benchmark configuration 5a: fcollect (paper section "Collective Operations": push, inner loop
 * over destinations).  Every PE q receives at dst_off + p*bytes_per_pe the block at src_off of
 * every PE p.  LDST: one grid, each source vector loaded once and stored to all PEs.  SDMA /
 * MEMCPY: npes*npes copies.  AUTO uses the cutover of n_wg on bytes_per_pe. */
int shm_launch_fcollect(shm_ctx *ctx, uint64_t dst_off, uint64_t src_off, size_t bytes_per_pe, int n_wg, int path);

/* collect (paper section "Collective Operations": push broadcast / collect / fcollect; OpenSHMEM
 * collect): PE p contributes nbytes_per_pe[p] bytes from src_off (host array of npes sizes, read
 * during the call); every PE's dst_off receives the blocks in PE order, block p at the sum of the
 * sizes before it.  Push by loads/stores, n_wg groups per PE.  SHM_ERANGE if the concatenation or
 * the largest source block leaves the heap, SHM_EINVAL on overlap. */
int shm_launch_collect(shm_ctx *ctx, uint64_t dst_off, uint64_t src_off, const size_t *nbytes_per_pe, int n_wg);

/* The reduction matrix (paper section "Collective Operations", reduction paragraph): min, max, sum,
 * product, and, or, xor over 8..64-bit integers; min, max, sum, product over float and double
 * (and/or/xor with a floating type: SHM_EINVAL).  Element i of every PE's dst_off becomes
 * x0[i] op x1[i] op ... in PE order; every PE duplicates the computation from one local and npes-1
 * remote vector loads (algo SHM_REDUCE_DUPLICATE), or -- the method the same section names for very
 * large reductions, algo SHM_REDUCE_SPLIT -- the vector is divided by address across PEs, each PE
 * folds its slice and pushes the result to every PE.  Both give the same bits.  Integer sums and
 * products wrap; min/max keep the earlier operand on ties.  Offsets 16-byte aligned.  n_wg is the
 * most groups per PE the launch may use: a long SPLIT reduction (slices of 6 MiB or more) asked of a
 * group per compute unit or more runs exactly that many in all, drawing pieces of the slices from
 * the counters long fcollects and broadcasts use (same rule for recorded launches). */
int shm_launch_reduce(shm_ctx *ctx, uint64_t dst_off, uint64_t src_off, size_t nelems, int dtype, int op, int n_wg, int algo);

/* Broadcast (paper section "Collective Operations": push, inner loop over destinations): every
 * PE's dst_off receives the n bytes at src_off of PE `root` (the root's own dst_off too).  LDST:
 * n_wg groups of the root store to all PEs from one grid on the team stream.  SDMA / MEMCPY: one
 * copy per destination.  AUTO by the cutover of n_wg on n. */
int shm_launch_broadcast(shm_ctx *ctx, uint64_t dst_off, uint64_t src_off, size_t n, int root, int n_wg, int path);

/* Device-side synchronisation among PEs (same section: every PE pushes an atomic increment to every
 * other PE's counter and waits on its own).  One grid of npes groups on the team stream, group p
 * acting as PE p.  shm_launch_sync_all: `rounds` syncs (with_quiet != 0: barriers = quiet + sync +
 * acquire); dev_ticks as for shm_launch_wg_put_timed.  shm_launch_barrier_exchange, a barrier that
 * data depends on: in round r < rounds <= npes PE p puts its n bytes at src_off into slot p
 * (dst_off + p*n) of PE (p+1+r) mod npes, all PEs meet in a device barrier, then p copies the slot
 * just filled for it (that of PE (p-1-r) mod npes) to acc_off + r*n. */
int shm_launch_sync_all(shm_ctx *ctx, int rounds, int with_quiet, uint64_t *dev_ticks);
int shm_launch_barrier_exchange(shm_ctx *ctx, uint64_t dst_off, uint64_t src_off, uint64_t acc_off, size_t n, int rounds);

/* Benchmark configuration 5b: float32 sum over PEs, operand order PE 0, 1, ..., npes-1 for every
 * element, so all PEs get bit-identical results.  DUPLICATE: every PE computes every element from
 * one local and npes-1 remote loads (paper section "Collective Operations", reduction paragraph).
 * SPLIT: PE q reduces the q-th share of the addresses and pushes it to all PEs (same section, the
 * remark on very large reductions; launch shape as for shm_launch_reduce).  Offsets 4-byte aligned
 * (16 for the vector path). */
int shm_launch_reduce_sum_f32(shm_ctx *ctx, uint64_t dst_off, uint64_t src_off, size_t nelems, int n_wg, int algo);

#ifdef __cplusplus
}
#endif
#endif /* SHM355_H */
