// Run-time row schedule of the matrix-core kernel: the arithmetic of its ticket queues, shared by
// the kernel (perq_mfma.hip) and by the host-side model that checks it (perq_schedule_selftest in
// perq_host.cpp).
//
// W workers (a wave on rows of its own, else a workgroup) share n_units units of work.  Worker w
// takes units w and w + W without asking anyone.  Every further unit belongs to one of kQueues
// queues: queue q owns units 2W + q + kQueues * t, t = 0 .. units_q - 1, and hands them out through
// a ticket counter that starts at zero.  A worker draws from the queue of its workgroup, takes the
// unit of every ticket below units_q, and stops at its first ticket at or past units_q.  A queue
// with workers_q workers therefore hands out exactly units_q + workers_q tickets per launch;
// whoever draws the last one, ticket units_q + workers_q - 1, stores zero, and the counter is ready
// for the next launch of the same stream.
#pragma once
#include <cstdint>

namespace perq {
namespace schedule {

constexpr uint32_t kQueues = 32;     // ticket counters per set
constexpr uint32_t kSets = 64;       // sets per device: one per stream that launches the kernel

struct QueuePlan {
    uint32_t first_unit;    // unit of ticket 0
    uint32_t units;         // units this queue hands out
    uint32_t last_ticket;   // the ticket whose drawer puts the counter back to zero
};

// queue of workgroup `block`: workgroups 8k .. 8k+7 (one per XCD) share a queue
__host__ __device__ inline uint32_t queue_of_block(uint32_t block) { return (block >> 3) & (kQueues - 1u); }

// The launch side guarantees n_blocks % (8 * kQueues) == 0 (every queue has the same number of
// workers, workers_per_block * n_blocks / kQueues of them) and n_units >= 2 * n_workers.
__host__ __device__ inline QueuePlan queue_plan(uint32_t n_units, uint32_t n_workers, uint32_t queue) {
    QueuePlan q;
    q.first_unit = 2u * n_workers + queue;
    q.units = n_units > q.first_unit ? (n_units - q.first_unit + kQueues - 1u) / kQueues : 0u;
    q.last_ticket = q.units + n_workers / kQueues - 1u;
    return q;
}

__host__ __device__ inline uint32_t unit_of_ticket(const QueuePlan& q, uint32_t ticket) {
    return q.first_unit + kQueues * ticket;
}

// whether a launch of n_blocks workgroups over n_units units may use the queues at all
__host__ __device__ inline bool queues_usable(int64_t n_blocks, int64_t n_workers, int64_t n_units) {
    return n_blocks % (8 * (int64_t)kQueues) == 0 && n_units >= 2 * n_workers;
}

}  // namespace schedule
}  // namespace perq
