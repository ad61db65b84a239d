// An application kernel of the kind the paper's section "Proposed Device APIs" is about: code that
// is NOT part of the library, includes only the device header, receives the device view that
// shm_device_context() hands out, and calls the OpenSHMEM operations from inside its own kernel.
// Built as a separate shared library (libshm355_user_example.so) that does not link the library.
//
// The first kernel is an all-to-all exchange with a device-side barrier and an atomic tally:
//   * one work-group per PE (blockIdx.x = PE p); block t of p's source goes to slot p of PE t's
//     destination with a work-group put (p's own block included);
//   * barrier_all_work_group: everybody's blocks have landed and are visible;
//   * every PE gets its right-hand neighbour's slot 0 (the block PE 0 sent there) into `back` with a
//     work-group get, and thread 0 adds p + 1 to a 64-bit tally on PE 0 with a fetch-add, storing
//     what it fetched to its own `seen` word.
// All npes groups must be resident together (they meet in the barrier); npes <= 32 groups always are.
#include <hip/hip_runtime.h>

#include <cstring>

#include "shm_device.hpp"

namespace {

__global__ __launch_bounds__(256) void shmu_alltoall_kernel(shm_dev_ctx c, uint64_t dst_off, uint64_t src_off, size_t n, uint64_t back_off,
                                                            uint64_t tally_off, uint64_t seen_off)
{
    const int me = blockIdx.x, npes = c.npes;
    for (int j = 0; j < npes; ++j) {
        int t = me + j;                       // own block first, then round the ring
        if (t >= npes) t -= npes;
        shmx_putmem_wg(c, me, dst_off + static_cast<uint64_t>(me) * n, src_off + static_cast<uint64_t>(t) * n, n, t);
    }
    shmx_barrier_all_wg(c, me);
    int right = me + 1;
    if (right >= npes) right -= npes;
    shmx_getmem_wg(c, me, back_off, dst_off, n, right);
    if (threadIdx.x == 0) {
        const int64_t before = shm_atomic_fetch_add(c, tally_off, me + 1, 0);
        *reinterpret_cast<int64_t *>(shm_ptr(c, seen_off, me)) = before;
    }
}

// The collectives called from inside a kernel, one work-group per PE: every PE's block gathered on
// every PE, two reductions over the PEs' sources (int32 sum, int16 min), and the root's block
// broadcast -- each a single device call ending in its own barrier.
__global__ __launch_bounds__(256) void shmu_collectives_kernel(shm_dev_ctx c, uint64_t gather_off, uint64_t src_off, size_t n, uint64_t sum_off,
                                                               uint64_t min_off, size_t nelems, uint64_t bcast_off, int root)
{
    const int me = blockIdx.x;
    shmx_fcollect_wg(c, me, gather_off, src_off, n);
    shmx_reduce_wg<int32_t, SHMD_OP_SUM>(c, me, sum_off, src_off, nelems);
    shmx_reduce_wg<int16_t, SHMD_OP_MIN>(c, me, min_off, src_off, 2 * nelems);
    shmx_broadcast_wg(c, me, bcast_off, src_off, n, root);
}

// A long message moved on group-owned tiles by groups of the caller's own size (the paper varies
// the work-items per work-group): gridDim.x groups of blockDim.x threads of PE `me` put n bytes
// to PE `pe`, then the same groups get them back from there into `back_off` of their own heap.
__global__ __launch_bounds__(1024) void shmu_tiles_kernel(shm_dev_ctx c, int me, int pe, uint64_t dst_off, uint64_t src_off, size_t n)
{
    shmx_putmem_tiles(c, me, dst_off, src_off, n, pe, blockIdx.x, gridDim.x);
}

__global__ __launch_bounds__(1024) void shmu_tiles_back_kernel(shm_dev_ctx c, int me, int pe, uint64_t dst_off, size_t n, uint64_t back_off)
{
    shmx_getmem_tiles(c, me, back_off, dst_off, n, pe, blockIdx.x, gridDim.x);
}

}  // namespace

extern "C" {

// Offsets 16-byte aligned; threads 1..1024; groups >= 1.  The get is a second kernel on the same
// stream, so it starts when every group of the put has finished.
int shmu_tiles(const void *devctx, size_t devctx_bytes, void *stream, int me, int pe, uint64_t dst_off, uint64_t src_off, size_t n,
               uint64_t back_off, int groups, int threads)
{
    if (!devctx || devctx_bytes != sizeof(shm_dev_ctx) || ((dst_off | src_off | back_off) & 15) || groups < 1 || threads < 1 || threads > 1024)
        return -1;
    shm_dev_ctx c;
    memcpy(&c, devctx, sizeof c);
    if (c.npes < 1 || c.npes > SHM_MAX_PES || me < 0 || me >= c.npes || pe < 0 || pe >= c.npes) return -1;
    hipLaunchKernelGGL(shmu_tiles_kernel, dim3(groups), dim3(threads), 0, static_cast<hipStream_t>(stream), c, me, pe, dst_off, src_off, n);
    if (hipGetLastError() != hipSuccess) return -5;
    hipLaunchKernelGGL(shmu_tiles_back_kernel, dim3(groups), dim3(threads), 0, static_cast<hipStream_t>(stream), c, me, pe, dst_off, n,
                       back_off);
    return hipGetLastError() == hipSuccess ? 0 : -5;
}

// devctx: HOST pointer to the bytes shm_device_context() wrote; stream: a hipStream_t.  Offsets are
// symmetric-heap byte offsets (tally_off and seen_off 8-byte aligned).  Returns 0, -1 for a view of
// the wrong size or bad arguments, -5 for a HIP error.  Asynchronous on `stream`.
int shmu_alltoall(const void *devctx, size_t devctx_bytes, void *stream, uint64_t dst_off, uint64_t src_off, size_t n, uint64_t back_off,
                  uint64_t tally_off, uint64_t seen_off)
{
    if (!devctx || devctx_bytes != sizeof(shm_dev_ctx) || ((tally_off | seen_off) & 7)) return -1;
    shm_dev_ctx c;
    memcpy(&c, devctx, sizeof c);
    if (c.npes < 1 || c.npes > SHM_MAX_PES) return -1;
    hipLaunchKernelGGL(shmu_alltoall_kernel, dim3(c.npes), dim3(256), 0, static_cast<hipStream_t>(stream), c, dst_off, src_off, n, back_off,
                       tally_off, seen_off);
    return hipGetLastError() == hipSuccess ? 0 : -5;
}

// n bytes per PE are gathered and broadcast; the first 4 * nelems of them are reduced.  Offsets 4-byte aligned.
int shmu_collectives(const void *devctx, size_t devctx_bytes, void *stream, uint64_t gather_off, uint64_t src_off, size_t n, uint64_t sum_off,
                     uint64_t min_off, size_t nelems, uint64_t bcast_off, int root)
{
    if (!devctx || devctx_bytes != sizeof(shm_dev_ctx) || ((src_off | sum_off | min_off) & 3) || 4 * nelems > n) return -1;
    shm_dev_ctx c;
    memcpy(&c, devctx, sizeof c);
    if (c.npes < 1 || c.npes > SHM_MAX_PES || root < 0 || root >= c.npes) return -1;
    hipLaunchKernelGGL(shmu_collectives_kernel, dim3(c.npes), dim3(256), 0, static_cast<hipStream_t>(stream), c, gather_off, src_off, n, sum_off,
                       min_off, nelems, bcast_off, root);
    return hipGetLastError() == hipSuccess ? 0 : -5;
}

size_t shmu_device_context_bytes(void) { return sizeof(shm_dev_ctx); }

}  // extern "C"
