// Device side of the scratch header: ticket queues that hand out tiles and the launch counter, the bounded
// wait for carry records, per-tile time stamps.  The layout of the header is described in
// heinsen_internal.hpp.
#pragma once
#include "heinsen_internal.hpp"
#include "heinsen_math.hpp"

namespace hs {

struct Draw {
    uint32_t ticket; // position in the queue's start order
    uint32_t epoch;  // launch counter, the tag of this launch's carry records
};

// One thread of a workgroup draws the workgroup's ticket from `queue`.  Every launch draws exactly
// `draws_per_queue` tickets from each of its `nqueues` queues (workgroups that find no tile behind their
// ticket simply end), so whoever draws a queue's last ticket knows that queue is finished for this launch,
// and whoever finishes the last queue re-arms all of them for the next launch with the next epoch.
__device__ __forceinline__ Draw draw_ticket(rec_t *header, int queue, uint32_t draws_per_queue, int nqueues)
{
    const rec_t old = __hip_atomic_fetch_add(header + kQueueStride * queue, 1ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    const Draw d{(uint32_t)old, (uint32_t)(old >> 32)};
    if (d.ticket + 1u == draws_per_queue) {
        bool all = true;
        if (nqueues > 1) {
            const rec_t done = __hip_atomic_fetch_add(header + kHeaderQueuesDone, 1ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            all = done + 1ull == (rec_t)nqueues;
            if (all) __hip_atomic_store(header + kHeaderQueuesDone, 0ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
        if (all) {
            const uint32_t next = d.epoch >= kLastEpoch ? 1u : d.epoch + 1u;
            for (int q = 0; q < kQueues; ++q)
                __hip_atomic_store(header + kQueueStride * q, (rec_t)next << 32, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
    } else if (d.ticket >= draws_per_queue) {
        // more draws than the launch has workgroups: two launches are using this scratch at once
        __hip_atomic_fetch_or(header + kHeaderError, 2ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    return d;
}

// Last action of every workgroup of a launch that drew tickets (all threads call it).  Only the launch that
// carries the last epoch does anything here: once all of its workgroups have ended, the last one clears
// the records, so that no tag of this cycle of epochs can be taken for one of the next cycle.
__device__ __forceinline__ void end_of_workgroup(rec_t *header, uint32_t epoch, uint32_t *s_flag)
{
    if (epoch != kLastEpoch) return;
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); // this wave's record stores have arrived
    __syncthreads();
    if (threadIdx.x == 0) {
        const rec_t n = __hip_atomic_fetch_add(header + kHeaderExited, 1ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        const bool last = n + 1ull == (rec_t)gridDim.x;
        if (last) __hip_atomic_store(header + kHeaderExited, 0ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        *s_flag = last ? 1u : 0u;
    }
    __syncthreads();
    if (*s_flag) {
        const size_t cap = (size_t)header[kHeaderCapacity];
        for (size_t i = kRecordBase + threadIdx.x; i < cap; i += blockDim.x)
            __hip_atomic_store(header + i, 0ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
}

// A tile that has polled `spin_limit` times without its carry records arriving gives up: it notes the fact
// in the header and goes on with NaN as its start state, which it also hands on, so that every workgroup
// ends and the damage shows in the output.  (Records can only stay away when two launches use one scratch
// at the same time, which the interface forbids.)
__device__ __forceinline__ void note_wait_gave_up(rec_t *header)
{
    __hip_atomic_fetch_or(header + kHeaderError, 1ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// Optional per-tile time stamps (a 100 MHz wall clock), eight per tile, written by the tile's first thread.
struct Timeline {
    unsigned long long *stamps;
    uint32_t tiles;
    __device__ __forceinline__ void mark(uint32_t tile, int slot) const
    {
        if (stamps != nullptr && tile < tiles && threadIdx.x == 0) stamps[(size_t)tile * 8 + slot] = wall_clock64();
    }
    __device__ __forceinline__ void mark_at(uint32_t tile, int slot, unsigned long long t) const
    {
        if (stamps != nullptr && tile < tiles && threadIdx.x == 0) stamps[(size_t)tile * 8 + slot] = t;
    }
};

} // namespace hs
