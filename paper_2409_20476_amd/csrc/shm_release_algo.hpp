// The protocol by which the work-groups of one XCD share their agent-scope releases, written once
// for both sides: the device instantiates it with agent-scope atomics on a word of the library's
// tail and the cache write-back as `write_back`; a CPU test instantiates it with std::atomic and
// threads and checks the property that makes it a quiet -- every caller returns only after a
// write-back that BEGAN after the caller arrived has finished -- under contention.  No HIP types
// here: the header compiles with any C++17 compiler.
//
// The word:  bit 0       set while one caller is writing back (the lock)
//            bits 63..1  number of shared write-backs that have FINISHED
// A caller sets bit 0 with one fetch-or.  If the bit was clear the caller is the one who writes back:
// write_back(), then ONE store that publishes count + 1 and clears the lock -- two memory round trips
// in all when nobody else is releasing.  If the bit was set, with count c, write-back c + 1 is under
// way and may have begun before this caller's stores arrived; the caller is covered by write-back
// c + 2, which can only begin after c + 1 has ended, i.e. after this moment.  The caller polls the
// word: count >= c + 2 ends the wait; a clear lock lets it try to become the one who writes back (if,
// once it holds the lock, the count shows that a covering write-back finished meanwhile, it only
// clears the lock).  The holder of the lock never waits for anybody, so every wait ends; waits are
// bounded all the same: a caller that has polled spin_limit times writes back for itself.
//
// Ops:  unsigned long long fetch_or_lock()   atomically set bit 0, return the word before
//       unsigned long long load()            the word now
//       void store(unsigned long long)       replace the word (only ever called by the lock's holder)
//       void write_back()                    complete everything that had arrived before the call
//       void pause()                         between polls
#pragma once

#if defined(__HIPCC__) || defined(__CUDACC__)
#define SHM_ALGO_FN __host__ __device__ inline
#else
#define SHM_ALGO_FN inline
#endif

template <typename Ops>
SHM_ALGO_FN void shm_release_shared_algo(Ops &ops, int spin_limit)
{
    unsigned long long v = ops.fetch_or_lock();
    if (!(v & 1ull)) {                         // nobody was writing back: this caller does, for everybody
        ops.write_back();
        ops.store(v + 2ull);                   // count + 1, lock clear
        return;
    }
    const unsigned long long need = (v >> 1) + 2ull;
    for (int spin = 0; spin < spin_limit; ++spin) {
        ops.pause();
        v = ops.load();
        if ((v >> 1) >= need) return;
        if (!(v & 1ull)) {
            v = ops.fetch_or_lock();
            if (!(v & 1ull)) {                 // the lock is ours
                if ((v >> 1) < need) {
                    ops.write_back();
                    v += 2ull;
                }
                ops.store(v);
                return;
            }
            if ((v >> 1) >= need) return;
        }
    }
    ops.write_back();                          // polled for too long: release without the others
}
