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
    std::vector<double> rate_after; // n clock speeds after the batch
    int64_t n_gossip = 0, n_grad = 0, n_grad_xi = 0, n_grad_c = 0, n_grad_h = 0;
};

// Pure host function behind a2cid_plan_batch and a2cid_apply_events.  scratch_* are
// reusable work arrays (resized as needed) so that repeated calls do not allocate.
struct PlanScratch {
    std::vector<int64_t> level_stamp;   // per worker: 1 + index of the last level that touched it
    std::vector<int64_t> last_op;       // per worker: index of its last op in the batch, or -1
};
// rate_now: the speed of every worker's own clock (a2cid_op.clock_rate), or NULL for all 1.
int plan_batch(const Graph &g, double eta, const double *t_now, const double *rate_now, const a2cid_event_batch *batch,
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

// ---- The resident kernel's programme for one launch (planner: a2cid_host.cpp, kernel: a2cid_kernels.hip.h) ----
// W waves share a tile of 64 * C columns that stays in LDS for the whole launch.  Each wave runs its own linear
// programme of 16-byte slots, typed by position:
//   control:   x = gossip operations | gradient operations << 8 that follow (a level: every wave passes a workgroup
//              barrier first), or kResJump (continue with the next set of 64 slots), or kResEnd; in the first slot of
//              a programme also y = ordinal of the wave's first gradient event (kResNone: it has none), z/w = that
//              event's xi
//   gossip:    x = LDS byte offset of row i, y = of row j, z = b_i, w = b_j (fp32 bits); with trailing mixes a second
//              slot follows: x = bp_i, y = bp_j
//   gradient:  two slots: x = LDS byte offset of the row, y = b_i, z = gamma, w = gscale; then x = ordinal of the
//              wave's next gradient event or kResNone, y = bp_i, z/w = xi of that next event (low, high word)
// A gradient input is a device pointer to the row, or an odd value, which is no pointer but stands for a constant
// row: 1 for zeros, 3 for ones.  Every wave's programme has the same number of level slots, a level never straddles
// a set of 64 slots, and a programme has at most resident_slots(W) slots including its end slot.
struct ResSlot { uint32_t x, y, z, w; };
static_assert(sizeof(ResSlot) == 16 && sizeof(ResSlot) == sizeof(a2cid_resident_slot), "ResSlot layout");
struct GradIn { uintptr_t xi, c, h; };
enum : uint32_t { kResJump = 0x10000u, kResEnd = 0x20000u };
constexpr uint32_t kResNone = 0xffffffffu;
constexpr uintptr_t kResZeros = 1u, kResOnes = 3u;
constexpr int kResSetMax = 62;           // operation slots of one wave between two control slots
// Slots of one wave's programme: sets of 64, one slot per lane and set.  Four sets (16 registers) when 16 waves share
// the operations of a level, eight otherwise (a wave then has twice the operations, and registers to spare).
constexpr int resident_sets(int waves) { return waves >= 16 ? 4 : 8; }
constexpr int resident_slots(int waves) { return 64 * resident_sets(waves); }
constexpr size_t resident_lds_bytes(int cols, int n_rows) { return (size_t)n_rows * 64 * 8 * (size_t)cols; }
constexpr uint32_t resident_row_bytes(int cols) { return 64u * 8u * (uint32_t)cols; }
constexpr int32_t kResidentMaxRows = 320;    // 512 bytes of the 160 KiB of LDS per row and column-per-lane

struct ResidentPlan {
    std::vector<std::vector<ResSlot>> programme;    // per wave
    std::vector<int32_t> rows;                      // LDS row -> worker, in order of first use
    std::vector<int64_t> grad_op;                   // gradient ordinal -> index of the event in the batch
    int32_t n_xi = 0, n_c = 0, n_h = 0;             // gradient inputs the launch reads
    // work arrays
    std::vector<int32_t> slot_of;                   // per worker: its LDS row or -1
    std::vector<int64_t> last_grad_slot;            // per wave: index of the second slot of its latest gradient operation
    std::vector<int32_t> last_grad_level;           // per wave: (sub-)level of its latest gradient event
    std::vector<int32_t> wave_load, wave_slots;     // per wave: operations / slots dealt to it in the current (sub-)level
    std::vector<int32_t> wave_of;                   // per operation of the current (sub-)level: its wave
};
// Launch shape for a batch: waves per tile = the smallest power of two (2 ... 16) with at most 1.6 operations of an
// average level per wave; columns per lane = as many (4, 2, 1) as still let 32 / waves workgroups share a CU's LDS.
void resident_shape(int32_t n, const a2cid_event_batch *batch, int *waves, int *cols);
// Writes the programmes of one launch: the operations of the batch from *k on (which lies in level *l), as many whole
// (sub-)levels as the programmes hold.  On return *l, *k name the first operation not included.  coef: the batch's
// coefficients (plan_batch); trailing: gossip operations take two slots.  The batch must be valid (plan_batch passed).
void plan_resident(int32_t n, const a2cid_event_batch *batch, const a2cid_coef *coef, int waves, int cols,
                   bool trailing, int32_t *l, int64_t *k, ResidentPlan &plan);

// ---- The register-file kernel's programme for one launch (planner: a2cid_host.cpp, kernel: a2cid_kernels.hip.h) ----
// One wave owns 64 columns and keeps its column of every worker's x and xt in vector registers for the whole launch
// (worker r in register r and 64 + r: at most kRegMaxRows workers).  All waves run the same linear programme of
// 16-byte slots, fetched with scalar loads in blocks of kRegBlock slots; a slot's kind is x >> 8:
//   gossip:    x = i, y = j, z = b_i, w = b_j (fp32 bits)
//   gradient:  x = i | kRegGradient << 8, y = b_i, z = gamma, w = gscale; its inputs are entry (ordinal % kRegChunk)
//              of the chunk of gradient inputs in use (the launch's gradient events in programme order, kRegChunk to
//              a chunk)
//   mix:       x = i | kRegMix << 8, y = b (a trailing mix, right after its operation)
//   control:   x = kRegControl << 8, y = kRegEnd (end of the programme), 0 (filler), or, in the first slot of a block
//              only, kRegSwitch / kRegRequest: a request block
// A request block names the inputs of one chunk: slots 1-4 hold the 8 xi pointers (two to a slot: x, y = low and high
// word of the first, z, w of the second), the rest is filler; with centres and curvatures (`full`) a second block
// follows with the c pointers in slots 0-3 and the h pointers in slots 4-7.  A pointer with bit 0 set is the address
// of one float that stands for every column (absent input, or an event past the last).  The programme begins with the
// request blocks of chunks 0 and 1 (kRegRequest); before the first gradient event of chunk k >= 1 comes the request
// block of chunk k + 1 (kRegSwitch): the kernel waits for chunk k's inputs, requests chunk k + 1 into the registers
// chunk k - 1 used, and turns to chunk k.
// Every operation slot is applied in order; any order that keeps each worker's own operations in sequence gives the
// same bits, and the planner keeps the batch's.
enum : uint32_t { kRegGossip = 0, kRegGradient = 1, kRegMix = 2, kRegControl = 3 };
enum : uint32_t { kRegSwitch = 1, kRegEnd = 2, kRegRequest = 3 };
constexpr int kRegBlock = 8;             // slots per scalar fetch
constexpr int kRegChunk = 8;             // gradient events per chunk of inputs (two chunks are held in registers)
constexpr int32_t kRegMaxRows = 64;

struct RegPlan {
    std::vector<ResSlot> programme;
    std::vector<int64_t> grad_op;       // gradient ordinal -> index of the event in the batch
    uint64_t touched = 0;               // bit r: worker r is read and written by the launch
    int32_t n_xi = 0, n_c = 0, n_h = 0; // gradient inputs the launch reads
    std::vector<size_t> request_at;     // work array: first slot of request block q
};
// Writes the programme for the operations of the batch from *k on, as many as max_slots slots hold (a multiple of
// kRegBlock; at least one block more than the first requests and the longest single operation need).  On return *k
// names the first operation not included.  full: request blocks carry c and h pointers (needed as soon as one event
// of the launch has a centre or a curvature with gscale != 0); zero_one: device address of a float 0 followed by a
// float 1.  The batch must be valid (plan_batch passed) and n <= kRegMaxRows.
void plan_regfile(int32_t n, const a2cid_event_batch *batch, const a2cid_coef *coef, int64_t max_slots, bool full,
                  uintptr_t zero_one, int64_t *k, RegPlan &plan);
// What the kernel relies on without testing it (indices below n, chunk sizes, block structure): checked before
// every launch, so that a planner mistake becomes an error instead of a wave addressing registers it does not own.
bool regfile_programme_ok(const std::vector<ResSlot> &prog, int32_t n, bool full);

}  // namespace a2cid
