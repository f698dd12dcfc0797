// Internal declarations shared by the host translation unit (planner, scheduler, graph
// quantities) and the HIP translation unit (context, kernels).  Not part of the public ABI.
#pragma once

#include <cstdarg>
#include <cstdint>
#include <vector>

#include "a2cid.h"

namespace a2cid {

// Sets the thread-local message returned by a2cid_last_error() and returns code.
int fail(int code, const char *fmt, ...) __attribute__((format(printf, 2, 3)));
void clear_error();

// Undirected graph copied out of an a2cid_graph, with an n x n adjacency bitmap for
// O(1) membership tests while validating gossip events.
struct Graph {
    int32_t n = 0;
    std::vector<int32_t> u, v;
    std::vector<double> rate;
    std::vector<uint8_t> adj;   // n * n, adj[i * n + j] == 1 iff {i, j} is an edge

    bool has_edge(int32_t i, int32_t j) const { return adj[(size_t)i * n + j] != 0; }
};

// Validates and copies.  Returns A2CID_OK / A2CID_EINVAL / A2CID_EGRAPH.
int load_graph(Graph &g, int32_t n, const a2cid_graph *src);

// Off-diagonal entry b of exp(tau [[-eta, eta], [eta, -eta]]) = [[1-b, b], [b, 1-b]]
// (closed form of the mixing step of Algorithm 1): b = (1 - exp(-2 eta tau)) / 2.
double mix_coefficient(double eta, double tau);

// Result of planning one batch (the validation + coefficient step, S3 of the path).
struct Plan {
    std::vector<a2cid_coef> coef;   // one per op
    std::vector<double> t_after;    // n time stamps after the batch
    int64_t n_gossip = 0, n_grad = 0, n_grad_xi = 0, n_grad_c = 0, n_grad_h = 0;
};

// Pure host function behind a2cid_plan_batch and a2cid_apply_events.  scratch_* are
// reusable work arrays (resized as needed) so that repeated calls do not allocate.
struct PlanScratch {
    std::vector<int64_t> level_stamp;   // per worker: 1 + index of the last level that touched it
    std::vector<int64_t> last_op;       // per worker: index of its last op in the batch, or -1
};
int plan_batch(const Graph &g, double eta, const double *t_now, const a2cid_event_batch *batch,
               Plan &plan, PlanScratch &scratch);

// The chain kernel's programme for one launch: the order in which the operations are applied and where every
// touched worker's columns come from and go to.  Any linear extension of the per-worker orders gives the same
// result bit for bit (operations on disjoint rows commute exactly); this one is built greedily so that an
// operation finds its workers close by as often as possible.  A worker's columns can be in device memory, in the
// workgroup's carry registers (from one operation to the very next), or parked in one of lds_slots LDS slots:
//   - next comes the free pending operation of a worker used by the previous operation, of one of the
//     kChainRecent last used workers, or of a parked worker, whichever misses the fewest rows (ties: in that
//     order); when there is none, the earliest operation not yet emitted (always free in a level-sorted batch);
//   - a worker that the next operation uses stays in the carry registers; another worker with a pending
//     operation is parked if a slot is free or holds a worker whose next operation comes later in the batch
//     (that worker is written back first: a spill step); everything else goes to memory;
//   - a worker is parked only while it has a pending operation and goes to memory after its last one, so
//     memory is complete when the launch ends.
struct ChainPlan {
    std::vector<a2cid_chain_step> steps;
    double bytes_per_column = 0.0;      // what the launch moves: 8 per row read from or written to memory, 4 per input
    // work arrays
    std::vector<int32_t> next_op;       // [2 k + e]: the next operation of operation k's endpoint e, or -1
    std::vector<int32_t> waiting;       // endpoints of operation k whose previous operation has not been emitted
    std::vector<int32_t> head;          // per worker: its first operation not yet emitted, or -1
    std::vector<int32_t> last;
    std::vector<int32_t> recent;        // workers in order of last use, most recent first
    std::vector<int32_t> owner;         // per LDS slot: the parked worker or -1
    std::vector<uint8_t> where;         // per worker: A2CID_LOC_* of its current columns
    std::vector<char> emitted;
};
constexpr size_t kChainRecent = 4;
constexpr int32_t kChainMaxSlots = 16;
// ops[0 .. count) must hold valid worker indices (0 <= i, j < n, i != j for gossip); 0 <= lds_slots <= kChainMaxSlots.
void plan_chain(int32_t n, const a2cid_op *ops, int64_t count, int32_t lds_slots, ChainPlan &plan);

}  // namespace a2cid
