// Context, launch logic and the GPU half of the C ABI (see include/a2cid.h).
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cmath>
#include <cstring>
#include <mutex>
#include <new>
#include <vector>

#include "a2cid_internal.h"
#include "a2cid_kernels.hip.h"

using namespace a2cid;

#define A2CID_HIP(call)                                                                      \
    do {                                                                                     \
        hipError_t e_ = (call);                                                              \
        if (e_ != hipSuccess)                                                                \
            return fail(A2CID_EHIP, "%s failed: %s (%s:%d)", #call, hipGetErrorString(e_),    \
                        __FILE__, __LINE__);                                                 \
    } while (0)

// Scratch of a2cid_stats_static: per-workgroup partial sums of the observables kernel, for callers that cannot
// allocate.  Every GPU the library runs on holds its own copy of this array, at its own address, until the process
// ends.  In host code the name below is only a handle: the address a kernel may use comes from hipGetSymbolAddress
// (static_scratch()), once per device.
constexpr size_t kStaticDoubles = 2048 * (2 * 64 + 2);      // 2048 workgroups x 64 workers: 2 129 920 bytes
static __device__ __align__(256) double scratch[kStaticDoubles];

namespace {

constexpr int kSlots = 4;               // operation-table staging buffers in flight
constexpr int64_t kSlotOps = 16384;     // operations per staging buffer (1 MiB)
constexpr int64_t kResRecords = 8192;   // slots of the resident kernel's per-wave programmes per staging buffer (16 waves x 512)
constexpr int kStatsBlocksMax = 8192;   // upper bound on workgroups of the observables kernel (grid-stride)

struct Slot {
    DevOp *host = nullptr;              // pinned
    DevOp *dev = nullptr;
    // resident kernel only: rows touched, compact operation records, gradient inputs in order
    int32_t *rows_host = nullptr, *rows_dev = nullptr;   // A2CID_MAX_WORKERS entries
    ResSlot *res_host = nullptr, *res_dev = nullptr;     // kResRecords entries
    GradIn *gin_host = nullptr, *gin_dev = nullptr;      // kSlotOps entries
    hipEvent_t done = nullptr;
    bool in_flight = false;
};

// Pinned staging for the n pending mixing coefficients that a2cid_stats and a2cid_average upload: two buffers, each
// guarded by an event, so that a call never has to wait for the stream before it may write the next set.
struct CoefStage {
    float *host = nullptr;              // pinned, n floats
    hipEvent_t done = nullptr;
    bool in_flight = false;
};

struct TimedLaunch {
    hipEvent_t start, stop;
};

struct DevSpan {
    uintptr_t lo, hi;                   // one device allocation, [lo, hi)
};
constexpr size_t kKnownSpans = 64;

}  // namespace

struct a2cid_ctx {
    Graph g;
    int32_t n = 0;
    int64_t d = 0, ld = 0;
    float *x = nullptr, *xt = nullptr;
    hipStream_t stream = nullptr;
    int device = -1;                    // the GPU that was current at creation and owns x, xt and the scratch
    std::vector<DevSpan> known;         // device allocations that passed check_device_span (a cache)
    double eta = 0, alpha = 0, alpha_t = 0;
    std::vector<double> t;
    std::vector<double> rate;           // speed of every worker's own clock against the event times (default 1)
    Plan plan;
    PlanScratch scratch;
    Slot slots[kSlots];
    int next_slot = 0;
    // launch shape of the level kernel (tunable through a2cid_set_tuning)
    int unroll = 1;
    int nontemporal = 0;
    int threads = 256;
    int walk = -1;                      // 0: one launch per level; 1: one walk launch per batch; 2: resident; 3: chain;
                                        // -1: 3, except 1 for very short rows (event_mode())
    int group = 0;                      // resident kernel: waves per workgroup (sharing one tile); 0: chosen per batch
    int group_now = 8, cols_now = 1;    // the shape of the launch being written
    float *zero_dev = nullptr;          // a zero float and, behind it, a one: stand in for absent gradient inputs
    int resident_cols = 1;              // resident kernel: columns per lane (1, 2 or 4) when group != 0
    int order = 0;                      // 0: jumps after the mixing (Eq. (1)); 1: Algorithm 1's listing order
    ResidentPlan resplan;               // resident kernel: the launch being planned
    RegPlan regplan;                    // register-file kernel: the launch being planned
    int stats_v = 2, stats_r = 2, stats_blocks = 2048, stats_nt = 1;   // launch shape of the observables kernel
    bool failed = false;                // an enqueueing step failed half-way: device state and time stamps disagree
    // observables scratch
    CoefStage coef_stage[2];
    int next_coef_stage = 0;
    float *b_dev = nullptr;
    double *partials = nullptr, *out_dev = nullptr, *out_host = nullptr;
    // counters since creation (or the last a2cid_counters_reset)
    int64_t n_gossip = 0, n_grad = 0, n_launch = 0;
    double alg_bytes = 0.0;
    double moved_bytes = 0.0;           // bytes the launched kernels move by construction (<= alg_bytes)
    ChainPlan chain;
    int chain_slots = 5;                // chain kernel: LDS slots for parked workers
    int walk_wg_per_cu = 0;             // walk kernel: at most this many workgroups per CU (0: whatever fits)
    // optional per-launch timing
    bool profiling = false;
    std::vector<TimedLaunch> timed;
    std::vector<TimedLaunch> timed_stats;   // the observables kernel, kept apart from the event kernels
    std::vector<hipEvent_t> event_pool;
};

namespace {

// Every call that touches the GPU must run with the context's device current: the scratch lives there and a
// launch on another device would hand its kernels pointers that device cannot reach.
int enter(const a2cid_ctx *c) {
    int dev = -1;
    A2CID_HIP(hipGetDevice(&dev));
    if (dev != c->device)
        return fail(A2CID_EINVAL, "the context belongs to HIP device %d but device %d is current", c->device, dev);
    return A2CID_OK;
}

int unusable(const a2cid_ctx *c) {
    if (!c->failed) return A2CID_OK;
    return fail(A2CID_EHIP, "the context is unusable: an earlier call failed after part of its work had been enqueued, "
                "so the device state and the time stamps no longer belong together");
}

// Turns a pointer that the kernels would fault on into an error: [p, p + bytes) has to be device (or managed)
// memory of the context's GPU and must not run past the end of its allocation.  Asks the runtime; allocates
// nothing.  On success *span (may be NULL) receives the extent of the allocation, or an empty span when the
// runtime knows the pointer but not its extent.  The check sees allocations, not tensors: a span that stays
// inside a larger allocation (a caching allocator's segment) passes.
int query_device_span(const a2cid_ctx *c, const void *p, size_t bytes, const char *what, DevSpan *span) {
    const uintptr_t lo = (uintptr_t)p, hi = lo + bytes;
    if (span) *span = DevSpan{0, 0};
    if (hi < lo) return fail(A2CID_EINVAL, "%s: %zu bytes from %p wrap the address space", what, bytes, p);
    hipPointerAttribute_t attr;
    std::memset(&attr, 0, sizeof(attr));
    if (hipPointerGetAttributes(&attr, p) != hipSuccess) {
        (void)hipGetLastError();
        return fail(A2CID_EINVAL, "%s: %p is not memory known to the HIP runtime (a host pointer?)", what, p);
    }
    if (attr.type != hipMemoryTypeDevice && attr.type != hipMemoryTypeManaged)
        return fail(A2CID_EINVAL, "%s: %p is not device memory", what, p);
    if (attr.type == hipMemoryTypeDevice && attr.device != c->device)
        return fail(A2CID_EINVAL, "%s: %p belongs to HIP device %d, the context to device %d", what, p, attr.device,
                    c->device);
    hipDeviceptr_t base = nullptr;
    size_t size = 0;
    if (hipMemGetAddressRange(&base, &size, (hipDeviceptr_t)p) != hipSuccess) {
        (void)hipGetLastError();
        return A2CID_OK;                // the runtime knows the pointer but not its extent: nothing more to check
    }
    const uintptr_t blo = (uintptr_t)base, bhi = blo + size;
    if (lo < blo || hi > bhi)
        return fail(A2CID_EINVAL, "%s: %zu bytes from %p run past the end of the allocation (%zu bytes at %p)", what,
                    bytes, p, size, (void *)base);
    if (span) *span = DevSpan{blo, bhi};
    return A2CID_OK;
}

// The same check with a memory: allocations that passed are remembered, so the runtime is asked once per
// allocation, not once per operation.  The memory lasts for one call of the library only (the caller of this
// function clears c->known first): an allocation freed and replaced between two calls is looked at again.
int check_device_span(a2cid_ctx *c, const void *p, size_t bytes, const char *what) {
    const uintptr_t lo = (uintptr_t)p, hi = lo + bytes;
    for (const DevSpan &k : c->known)
        if (k.lo <= lo && lo <= hi && hi <= k.hi) return A2CID_OK;
    DevSpan span;
    if (int rc = query_device_span(c, p, bytes, what, &span)) return rc;
    if (span.hi > span.lo) {
        if (c->known.size() >= kKnownSpans) c->known.clear();
        c->known.push_back(span);
    }
    return A2CID_OK;
}

// The address of this device's copy of the static scratch array.  Looked up once per device, with that device
// current (every caller has made sure of that), and kept.
constexpr int kMaxDevices = 64;
int static_scratch(int device, double **out) {
    static std::mutex guard;
    static double *address[kMaxDevices] = {};
    if (device < 0 || device >= kMaxDevices) return fail(A2CID_EINVAL, "HIP device %d out of range", device);
    std::lock_guard<std::mutex> lock(guard);
    if (!address[device]) {
        double *p = nullptr;
        A2CID_HIP(hipGetSymbolAddress((void **)&p, HIP_SYMBOL(scratch)));
        if (!p) return fail(A2CID_EHIP, "hipGetSymbolAddress returned a null address for the static scratch");
        address[device] = p;
    }
    *out = address[device];
    return A2CID_OK;
}

int acquire_coef_stage(a2cid_ctx *c, CoefStage **out) {
    CoefStage &s = c->coef_stage[c->next_coef_stage];
    c->next_coef_stage ^= 1;
    if (s.in_flight) {
        A2CID_HIP(hipEventSynchronize(s.done));
        s.in_flight = false;
    }
    *out = &s;
    return A2CID_OK;
}

int acquire_slot(a2cid_ctx *c, Slot **out) {
    Slot &s = c->slots[c->next_slot];
    c->next_slot = (c->next_slot + 1) % kSlots;
    if (s.in_flight) {
        A2CID_HIP(hipEventSynchronize(s.done));
        s.in_flight = false;
    }
    *out = &s;
    return A2CID_OK;
}

int get_event(a2cid_ctx *c, hipEvent_t *e) {
    if (!c->event_pool.empty()) {
        *e = c->event_pool.back();
        c->event_pool.pop_back();
        return A2CID_OK;
    }
    A2CID_HIP(hipEventCreate(e));
    return A2CID_OK;
}

enum LaunchKind { kLaunchLevel = 0, kLaunchWalk = 1, kLaunchChain = 3 };

template <int U, bool NT, int TPB>
void launch_t(a2cid_ctx *c, const DevOp *ops, int32_t n_ops, LaunchKind walk) {
    const int64_t n4 = c->d >> 2;
    const int64_t per_block = (int64_t)U * TPB;
    int64_t blocks = (n4 + per_block - 1) / per_block;
    if (blocks < 1) blocks = 1;   // the scalar tail lives in tile 0
    if (walk == kLaunchChain) {
        const size_t lds = (size_t)c->chain_slots * U * TPB * 2 * sizeof(v4f);
        if (lds > 65536)
            (void)hipFuncSetAttribute((const void *)chain_kernel<U, TPB>, hipFuncAttributeMaxDynamicSharedMemorySize,
                                      (int)lds);      // a failure shows as the launch error that follows
        hipLaunchKernelGGL((chain_kernel<U, TPB>), dim3((unsigned)blocks), dim3(TPB), lds, c->stream, c->x,
                           c->xt, c->ld, c->d, ops, n_ops, (float)c->alpha, (float)c->alpha_t);
    } else if (walk == kLaunchWalk) {
        // the kernel uses no LDS: asking for 1 / k of the CU's 160 KiB keeps at most k workgroups on a CU
        const size_t lds = c->walk_wg_per_cu > 0 ? (size_t)(160 * 1024) / c->walk_wg_per_cu - 256 : 0;
        if (lds > 65536)
            (void)hipFuncSetAttribute((const void *)walk_kernel<U, NT, TPB>, hipFuncAttributeMaxDynamicSharedMemorySize,
                                      (int)lds);      // a failure shows as the launch error that follows
        hipLaunchKernelGGL((walk_kernel<U, NT, TPB>), dim3((unsigned)blocks), dim3(TPB), lds, c->stream, c->x,
                           c->xt, c->ld, c->d, ops, n_ops, (float)c->alpha, (float)c->alpha_t);
    } else {
        hipLaunchKernelGGL((level_kernel<U, NT, TPB>), dim3((unsigned)blocks, (unsigned)n_ops), dim3(TPB), 0,
                           c->stream, c->x, c->xt, c->ld, c->d, ops, (float)c->alpha, (float)c->alpha_t);
    }
}

template <int U, bool NT>
void launch_u(a2cid_ctx *c, const DevOp *ops, int32_t n_ops, LaunchKind walk) {
    int threads = c->threads;
    while (threads > 64 && (c->d >> 2) / ((int64_t)U * threads) < 2048) threads >>= 1;
    switch (threads) {
        case 64: launch_t<U, NT, 64>(c, ops, n_ops, walk); break;
        case 128: launch_t<U, NT, 128>(c, ops, n_ops, walk); break;
        case 512: launch_t<U, NT, 512>(c, ops, n_ops, walk); break;
        case 1024: launch_t<U, NT, 1024>(c, ops, n_ops, walk); break;
        default: launch_t<U, NT, 256>(c, ops, n_ops, walk); break;
    }
}

// Enqueues n_ops operations: as one level (they must touch disjoint rows) or as a walk in order.
int launch_ops(a2cid_ctx *c, const DevOp *ops, int32_t n_ops, LaunchKind walk) {
    TimedLaunch tl{};
    if (c->profiling) {
        if (int rc = get_event(c, &tl.start)) return rc;
        if (int rc = get_event(c, &tl.stop)) return rc;
        A2CID_HIP(hipEventRecord(tl.start, c->stream));
    }
    const bool nt = c->nontemporal != 0 && walk != kLaunchChain;   // the chain kernel has one access policy
    // short rows: shrink the tile so that the grid still has a few thousand workgroups
    int unroll = c->unroll;
    while (unroll > 1 && (c->d >> 2) / ((int64_t)unroll * c->threads) < 2048) unroll >>= 1;
    switch (unroll) {
        case 1: nt ? launch_u<1, true>(c, ops, n_ops, walk) : launch_u<1, false>(c, ops, n_ops, walk); break;
        case 2: nt ? launch_u<2, true>(c, ops, n_ops, walk) : launch_u<2, false>(c, ops, n_ops, walk); break;
        default: nt ? launch_u<4, true>(c, ops, n_ops, walk) : launch_u<4, false>(c, ops, n_ops, walk); break;
    }
    A2CID_HIP(hipGetLastError());
    if (c->profiling) {
        A2CID_HIP(hipEventRecord(tl.stop, c->stream));
        c->timed.push_back(tl);
    }
    ++c->n_launch;
    return A2CID_OK;
}



// The resident kernel: flags of the launch are template cases.
template <int W, int C>
void launch_resident_wc(a2cid_ctx *c, const Slot *s, int32_t n_rows, unsigned blocks, size_t lds, bool pre,
                         bool trail, bool hc, bool hh, hipError_t *err) {
    *err = hipSuccess;
#define A2CID_RES(PRE, TRAIL, HC, HH)                                                                                    \
    do {                                                                                                             \
        if (lds > 65536)                                                                                             \
            *err = hipFuncSetAttribute((const void *)resident_kernel<W, C, PRE, TRAIL, HC, HH>,                    \
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);                        \
        if (*err == hipSuccess)                                                                                      \
            hipLaunchKernelGGL((resident_kernel<W, C, PRE, TRAIL, HC, HH>), dim3(blocks), dim3(64 * W), lds,       \
                               c->stream, c->x, c->xt, c->ld, c->d, s->res_dev, s->gin_dev,          \
                               s->rows_dev, n_rows, (float)c->alpha, (float)c->alpha_t);                             \
    } while (0)
    const int key = (pre ? 8 : 0) | (trail ? 4 : 0) | (hc ? 2 : 0) | (hh ? 1 : 0);
    switch (key) {
        case 0: A2CID_RES(false, false, false, false); break;
        case 1: A2CID_RES(false, false, false, true); break;
        case 2: A2CID_RES(false, false, true, false); break;
        case 3: A2CID_RES(false, false, true, true); break;
        case 4: A2CID_RES(false, true, false, false); break;
        case 5: A2CID_RES(false, true, false, true); break;
        case 6: A2CID_RES(false, true, true, false); break;
        case 7: A2CID_RES(false, true, true, true); break;
        case 8: A2CID_RES(true, false, false, false); break;
        case 9: A2CID_RES(true, false, false, true); break;
        case 10: A2CID_RES(true, false, true, false); break;
        case 11: A2CID_RES(true, false, true, true); break;
        case 12: A2CID_RES(true, true, false, false); break;
        case 13: A2CID_RES(true, true, false, true); break;
        case 14: A2CID_RES(true, true, true, false); break;
        default: A2CID_RES(true, true, true, true); break;
    }
#undef A2CID_RES
}

int launch_resident(a2cid_ctx *c, const Slot *s, int32_t n_rows, bool trailing, bool has_c, bool has_h) {
    TimedLaunch tl{};
    if (c->profiling) {
        if (int rc = get_event(c, &tl.start)) return rc;
        if (int rc = get_event(c, &tl.stop)) return rc;
        A2CID_HIP(hipEventRecord(tl.start, c->stream));
    }
    const int cols = c->cols_now;
    const unsigned blocks = (unsigned)((c->d + 64 * cols - 1) / (64 * cols));
    const size_t lds = resident_lds_bytes(cols, n_rows);
    if (lds > 160 * 1024) return fail(A2CID_EINVAL, "internal: %d rows x %d columns per lane exceed the LDS", n_rows, cols);
    hipError_t err = hipSuccess;
    const bool pre = c->order != 0;
    switch (c->group_now * 10 + cols) {
        case 11: launch_resident_wc<1, 1>(c, s, n_rows, blocks, lds, pre, trailing, has_c, has_h, &err); break;
        case 21: launch_resident_wc<2, 1>(c, s, n_rows, blocks, lds, pre, trailing, has_c, has_h, &err); break;
        case 22: launch_resident_wc<2, 2>(c, s, n_rows, blocks, lds, pre, trailing, has_c, has_h, &err); break;
        case 24: launch_resident_wc<2, 4>(c, s, n_rows, blocks, lds, pre, trailing, has_c, has_h, &err); break;
        case 41: launch_resident_wc<4, 1>(c, s, n_rows, blocks, lds, pre, trailing, has_c, has_h, &err); break;
        case 42: launch_resident_wc<4, 2>(c, s, n_rows, blocks, lds, pre, trailing, has_c, has_h, &err); break;
        case 44: launch_resident_wc<4, 4>(c, s, n_rows, blocks, lds, pre, trailing, has_c, has_h, &err); break;
        case 81: launch_resident_wc<8, 1>(c, s, n_rows, blocks, lds, pre, trailing, has_c, has_h, &err); break;
        case 82: launch_resident_wc<8, 2>(c, s, n_rows, blocks, lds, pre, trailing, has_c, has_h, &err); break;
        case 84: launch_resident_wc<8, 4>(c, s, n_rows, blocks, lds, pre, trailing, has_c, has_h, &err); break;
        case 161: launch_resident_wc<16, 1>(c, s, n_rows, blocks, lds, pre, trailing, has_c, has_h, &err); break;
        case 162: launch_resident_wc<16, 2>(c, s, n_rows, blocks, lds, pre, trailing, has_c, has_h, &err); break;
        case 164: launch_resident_wc<16, 4>(c, s, n_rows, blocks, lds, pre, trailing, has_c, has_h, &err); break;
        default: return fail(A2CID_EINVAL, "no resident kernel for %d waves and %d columns per lane", c->group_now, cols);
    }
    A2CID_HIP(err);
    A2CID_HIP(hipGetLastError());
    if (c->profiling) {
        A2CID_HIP(hipEventRecord(tl.stop, c->stream));
        c->timed.push_back(tl);
    }
    ++c->n_launch;
    return A2CID_OK;
}

// One launch of resident_kernel: plans the per-wave programmes for the operations of the batch from operation *k on
// (which lies in level *l), as many whole (sub-)levels as the programmes hold (plan_resident), uploads them and launches
// the kernel.  On return *l, *k name the first operation not included.
int enqueue_resident(a2cid_ctx *c, const a2cid_event_batch *batch, int32_t *l, int64_t *k, bool trailing) {
    Slot *s;
    if (int rc = acquire_slot(c, &s)) return rc;
    const int W = c->group_now;
    const int64_t k_before = *k;
    plan_resident(c->n, batch, c->plan.coef.data(), W, c->cols_now, trailing, l, k, c->resplan);
    if (*k == k_before) return fail(A2CID_EINVAL, "internal: a level does not fit an empty resident programme");
    const ResidentPlan &rp = c->resplan;
    const size_t per_wave = (size_t)resident_slots(W);
    const int32_t n_rows = (int32_t)rp.rows.size(), n_grad = (int32_t)rp.grad_op.size();
    if ((int64_t)(per_wave * (size_t)W) > kResRecords || n_rows > A2CID_MAX_WORKERS || n_grad > kSlotOps)
        return fail(A2CID_EINVAL, "internal: resident plan exceeds its staging buffers");
    for (int w = 0; w < W; ++w)
        std::memcpy(s->res_host + (size_t)w * per_wave, rp.programme[(size_t)w].data(), per_wave * sizeof(ResSlot));
    std::copy(rp.rows.begin(), rp.rows.end(), s->rows_host);
    for (int32_t g = 0; g < n_grad; ++g) {
        const a2cid_op &op = batch->ops[rp.grad_op[(size_t)g]];
        const bool affine = op.gscale != 0.f;
        s->gin_host[g].xi = op.xi ? (uintptr_t)op.xi : kResZeros;
        s->gin_host[g].c = (op.c && affine) ? (uintptr_t)op.c : kResZeros;
        s->gin_host[g].h = (op.h && affine) ? (uintptr_t)op.h : kResOnes;
    }
    A2CID_HIP(hipMemcpyAsync(s->rows_dev, s->rows_host, sizeof(int32_t) * (size_t)n_rows, hipMemcpyHostToDevice, c->stream));
    A2CID_HIP(hipMemcpyAsync(s->res_dev, s->res_host, sizeof(ResSlot) * per_wave * (size_t)W, hipMemcpyHostToDevice,
                             c->stream));
    if (n_grad > 0)
        A2CID_HIP(hipMemcpyAsync(s->gin_dev, s->gin_host, sizeof(GradIn) * (size_t)n_grad, hipMemcpyHostToDevice, c->stream));
    c->moved_bytes += (double)c->d * (16.0 * n_rows + 4.0 * (rp.n_xi + rp.n_c + rp.n_h));
    if (int rc = launch_resident(c, s, n_rows, trailing, rp.n_c > 0, rp.n_h > 0)) return rc;
    A2CID_HIP(hipEventRecord(s->done, c->stream));
    s->in_flight = true;
    return A2CID_OK;
}

// One launch of regfile_kernel: writes the programme for the operations of the batch from operation *k on, as many as
// a staging buffer holds (plan_regfile), uploads it and launches the kernel.  On return *k names the first operation
// not included.  full: some gradient event of the batch has a centre or a curvature; curvatures: some has a curvature.
int enqueue_regfile(a2cid_ctx *c, const a2cid_event_batch *batch, bool full, bool curvatures, int64_t *k) {
    Slot *s;
    if (int rc = acquire_slot(c, &s)) return rc;
    const int64_t k_before = *k;
    plan_regfile(c->n, batch, c->plan.coef.data(), kResRecords, full, (uintptr_t)c->zero_dev, k, c->regplan);
    if (*k == k_before) return fail(A2CID_EINVAL, "internal: an operation does not fit an empty register-file programme");
    const RegPlan &rp = c->regplan;
    if ((int64_t)rp.programme.size() > kResRecords || !regfile_programme_ok(rp.programme, c->n, full))
        return fail(A2CID_EINVAL, "internal: register-file programme of %zu slots fails its check", rp.programme.size());
    std::memcpy(s->res_host, rp.programme.data(), rp.programme.size() * sizeof(ResSlot));
    A2CID_HIP(hipMemcpyAsync(s->res_dev, s->res_host, sizeof(ResSlot) * rp.programme.size(), hipMemcpyHostToDevice,
                             c->stream));
    const int n_rows = __builtin_popcountll(rp.touched);
    c->moved_bytes += (double)c->d * (16.0 * n_rows + 4.0 * (rp.n_xi + rp.n_c + rp.n_h));
    TimedLaunch tl{};
    if (c->profiling) {
        if (int rc = get_event(c, &tl.start)) return rc;
        if (int rc = get_event(c, &tl.stop)) return rc;
        A2CID_HIP(hipEventRecord(tl.start, c->stream));
    }
    const unsigned blocks = (unsigned)((c->d + 63) / 64);
#define A2CID_REG(PRE, VARIANT)                                                                                         \
    hipLaunchKernelGGL((regfile_kernel<PRE, VARIANT>), dim3(blocks), dim3(64), 0, c->stream, c->x, c->xt, c->ld, c->d, \
                       s->res_dev, (uint32_t)(rp.programme.size() * sizeof(ResSlot)), rp.touched, (float)c->alpha,      \
                       (float)c->alpha_t)
    // centres only (two blocks per request, the curvature pointers unused) leave room for three waves per SIMD
    const int variant = !full ? 0 : curvatures ? 2 : 1;
    switch ((c->order != 0 ? 3 : 0) + variant) {
        case 0: A2CID_REG(false, 0); break;
        case 1: A2CID_REG(false, 1); break;
        case 2: A2CID_REG(false, 2); break;
        case 3: A2CID_REG(true, 0); break;
        case 4: A2CID_REG(true, 1); break;
        default: A2CID_REG(true, 2); break;
    }
#undef A2CID_REG
    A2CID_HIP(hipGetLastError());
    if (c->profiling) {
        A2CID_HIP(hipEventRecord(tl.stop, c->stream));
        c->timed.push_back(tl);
    }
    ++c->n_launch;
    A2CID_HIP(hipEventRecord(s->done, c->stream));
    s->in_flight = true;
    return A2CID_OK;
}

// Mixing every worker whose coefficient is non-zero, as one level of mix-only operations.
int enqueue_mix_all(a2cid_ctx *c, const std::vector<float> &b) {
    int32_t done = 0;
    while (done < c->n) {
        Slot *s;
        if (int rc = acquire_slot(c, &s)) return rc;
        int32_t count = 0;
        for (; done < c->n && count < kSlotOps; ++done) {
            if (b[done] == 0.f) continue;
            DevOp &o = s->host[count++];
            std::memset(&o, 0, sizeof(o));
            o.kind = kOpMixOnly;
            o.row_i = done;
            o.b_i = b[done];
        }
        if (count == 0) continue;
        A2CID_HIP(hipMemcpyAsync(s->dev, s->host, sizeof(DevOp) * (size_t)count, hipMemcpyHostToDevice, c->stream));
        if (int rc = launch_ops(c, s->dev, count, kLaunchLevel)) return rc;
        A2CID_HIP(hipEventRecord(s->done, c->stream));
        s->in_flight = true;
        c->alg_bytes += 16.0 * (double)c->d * count;
        c->moved_bytes += 16.0 * (double)c->d * count;
    }
    return A2CID_OK;
}

}  // namespace

extern "C" {

void a2cid_destroy(a2cid_ctx *c) {
    if (!c) return;
    (void)hipStreamSynchronize(c->stream);
    for (Slot &s : c->slots) {
        if (s.host) (void)hipHostFree(s.host);
        if (s.dev) (void)hipFree(s.dev);
        if (s.rows_host) (void)hipHostFree(s.rows_host);
        if (s.rows_dev) (void)hipFree(s.rows_dev);
        if (s.res_host) (void)hipHostFree(s.res_host);
        if (s.res_dev) (void)hipFree(s.res_dev);
        if (s.gin_host) (void)hipHostFree(s.gin_host);
        if (s.gin_dev) (void)hipFree(s.gin_dev);
        if (s.done) (void)hipEventDestroy(s.done);
    }
    for (CoefStage &cs : c->coef_stage) {
        if (cs.host) (void)hipHostFree(cs.host);
        if (cs.done) (void)hipEventDestroy(cs.done);
    }
    if (c->b_dev) (void)hipFree(c->b_dev);
    if (c->partials) (void)hipFree(c->partials);
    if (c->out_dev) (void)hipFree(c->out_dev);
    if (c->out_host) (void)hipHostFree(c->out_host);
    if (c->zero_dev) (void)hipFree(c->zero_dev);
    for (TimedLaunch &tl : c->timed) { (void)hipEventDestroy(tl.start); (void)hipEventDestroy(tl.stop); }
    for (TimedLaunch &tl : c->timed_stats) { (void)hipEventDestroy(tl.start); (void)hipEventDestroy(tl.stop); }
    for (hipEvent_t e : c->event_pool) (void)hipEventDestroy(e);
    delete c;
}

static int create_impl(a2cid_ctx *c, int32_t n, int64_t d, const a2cid_graph *graph, double eta,
                       double alpha, double alpha_tilde, const a2cid_buffers *buf) {
    if (int rc = load_graph(c->g, n, graph)) return rc;
    if (d < 1) return fail(A2CID_EINVAL, "d = %lld must be >= 1", (long long)d);
    if (!buf || !buf->x || !buf->xt) return fail(A2CID_EINVAL, "state buffers are NULL");
    if (buf->x == buf->xt) return fail(A2CID_EINVAL, "x and xt must be distinct buffers");
    if (buf->ld < d) return fail(A2CID_EINVAL, "ld = %lld is smaller than d = %lld", (long long)buf->ld, (long long)d);
    if ((buf->ld & 3) || ((uintptr_t)buf->x & 15u) || ((uintptr_t)buf->xt & 15u))
        return fail(A2CID_EALIGN, "x, xt must be 16-byte aligned and ld a multiple of 4");
    if (!(eta >= 0.0) || !std::isfinite(eta) || !std::isfinite(alpha) || !std::isfinite(alpha_tilde))
        return fail(A2CID_EINVAL, "eta must be finite and >= 0, alpha and alpha_tilde finite");
    c->n = n; c->d = d; c->ld = buf->ld;
    A2CID_HIP(hipGetDevice(&c->device));
    const size_t state_bytes = sizeof(float) * ((size_t)(n - 1) * (size_t)buf->ld + (size_t)d);
    if (int rc = check_device_span(c, buf->x, state_bytes, "x")) return rc;
    if (int rc = check_device_span(c, buf->xt, state_bytes, "xt")) return rc;
    c->x = buf->x; c->xt = buf->xt;
    c->stream = (hipStream_t)buf->hip_stream;
    c->eta = eta; c->alpha = alpha; c->alpha_t = alpha_tilde;
    c->t.assign(n, 0.0);
    c->rate.assign(n, 1.0);
    for (Slot &s : c->slots) {
        A2CID_HIP(hipHostMalloc((void **)&s.host, sizeof(DevOp) * kSlotOps, hipHostMallocDefault));
        A2CID_HIP(hipMalloc((void **)&s.dev, sizeof(DevOp) * kSlotOps));
        A2CID_HIP(hipHostMalloc((void **)&s.rows_host, sizeof(int32_t) * A2CID_MAX_WORKERS, hipHostMallocDefault));
        A2CID_HIP(hipMalloc((void **)&s.rows_dev, sizeof(int32_t) * A2CID_MAX_WORKERS));
        A2CID_HIP(hipHostMalloc((void **)&s.res_host, sizeof(ResSlot) * kResRecords, hipHostMallocDefault));
        A2CID_HIP(hipMalloc((void **)&s.res_dev, sizeof(ResSlot) * kResRecords));
        A2CID_HIP(hipHostMalloc((void **)&s.gin_host, sizeof(GradIn) * kSlotOps, hipHostMallocDefault));
        A2CID_HIP(hipMalloc((void **)&s.gin_dev, sizeof(GradIn) * kSlotOps));
        A2CID_HIP(hipEventCreateWithFlags(&s.done, hipEventDisableTiming));
    }
    const size_t m = 2 * (size_t)n + 2;
    for (CoefStage &cs : c->coef_stage) {
        A2CID_HIP(hipHostMalloc((void **)&cs.host, sizeof(float) * n, hipHostMallocDefault));
        A2CID_HIP(hipEventCreateWithFlags(&cs.done, hipEventDisableTiming));
    }
    A2CID_HIP(hipMalloc((void **)&c->b_dev, sizeof(float) * n));
    A2CID_HIP(hipMalloc((void **)&c->partials, sizeof(double) * m * kStatsBlocksMax));
    A2CID_HIP(hipMalloc((void **)&c->out_dev, sizeof(double) * m));
    A2CID_HIP(hipHostMalloc((void **)&c->out_host, sizeof(double) * m, hipHostMallocDefault));
    A2CID_HIP(hipMalloc((void **)&c->zero_dev, 256));
    A2CID_HIP(hipMemset(c->zero_dev, 0, 256));
    const float one = 1.f;
    A2CID_HIP(hipMemcpy(c->zero_dev + 1, &one, sizeof(one), hipMemcpyHostToDevice));
    double *static_ptr = nullptr;       // resolved here so that a2cid_stats_static never has to look it up
    if (int rc = static_scratch(c->device, &static_ptr)) return rc;
    return A2CID_OK;
}

int a2cid_create(a2cid_ctx **out, int32_t n, int64_t d, const a2cid_graph *graph, double eta,
                 double alpha, double alpha_tilde, const a2cid_buffers *buf) {
    clear_error();
    if (!out) return fail(A2CID_EINVAL, "out is NULL");
    *out = nullptr;
    a2cid_ctx *c = new (std::nothrow) a2cid_ctx;
    if (!c) return fail(A2CID_ENOMEM, "out of host memory");
    int rc;
    try {
        rc = create_impl(c, n, d, graph, eta, alpha, alpha_tilde, buf);
    } catch (const std::bad_alloc &) {
        rc = fail(A2CID_ENOMEM, "out of host memory");
    }
    if (rc != A2CID_OK) {
        // keep the message of the failure: a2cid_destroy makes HIP calls but never touches it
        a2cid_destroy(c);
        return rc;
    }
    *out = c;
    return A2CID_OK;
}

// The event kernel of the next batch when the choice is left to the library, from measurements (events per second,
// 1024 events per batch).  Up to 64 workers the register-file kernel: 1.4 to 2.0 times the LDS-resident kernel on
// the 64-worker configurations.  The LDS-resident kernel for up to 160 workers, the most for which two workgroups
// share a CU's LDS: with rows of 4 M parameters, ring / exponential graph, it is, against the chain kernel: 96 workers
// 1.4, 112: 2.3, 128: 1.4 / 2.4, 160: 1.3 times; from 192 workers on it depends on the graph (192 exponential 1.4,
// 256 ring 0.8, 256 exponential 1.4, 320 ring 0.8, 320 complete 1.5 times), so beyond 160 workers the chain kernel
// runs, or, for rows of at most 4096 parameters, the walk kernel (it needs no programme from the host).  Asked for
// explicitly, the resident kernel takes up to kResidentMaxRows workers.
constexpr int64_t kShortRow = 4096;
constexpr int32_t kResidentAutoRows = 160;
constexpr int64_t kRegMaxColumns = (int64_t)1 << 29;    // a lane's byte offset into a row stays below 2^31
static int event_mode(const a2cid_ctx *c) {
    if (c->walk >= 0) return c->walk;
    if (c->n <= kRegMaxRows && c->d <= kRegMaxColumns) return 4;
    if (c->n <= kResidentAutoRows) return 2;
    return c->d <= kShortRow ? 1 : 3;
}
// Operations per staging buffer: the chain programme of k operations has at most 3 k + slots steps (every spill makes
// room for a parking); the resident kernel's launches are cut to the size of its programmes on the way.
static int64_t piece_capacity(const a2cid_ctx *c) {
    switch (event_mode(c)) {
        case 3: return (kSlotOps - kChainMaxSlots) / 3;
        case 2: return kSlotOps;        // cut into launches on the way (enqueue_resident)
        default: return kSlotOps;
    }
}

static int enqueue_batch(a2cid_ctx *c, const a2cid_event_batch *batch);

// Launch shape of the resident kernel for a batch, unless the caller has fixed it: resident_shape (a2cid_host.cpp).
// Waves per tile: the smallest power of two with at most 1.6 operations of an average level per wave (more waves only
// add waves that pass the barrier with nothing to do; fewer make a level as long as several operations).  Columns per lane: as many as still let 32 / waves workgroups share a CU's 160 KiB of LDS (32 waves per CU
// is the hardware limit), at 512 bytes per row and column-per-lane.  Measured on the 64-worker configurations (events
// per second, 1024 events per batch): ring, 17.5 operations per level: 16 waves x 2 columns 108 k, 8 x 1 94 k;
// exponential graph, 11.5: 8 x 1 46.8 k, 16 x 2 44.6 k; complete graph, 10.1: 8 x 1 44.8 k, 16 x 2 41.6 k; 16 workers
// on a ring, 5.7: 4 x 2 766 k, 8 x 2 699 k.
static void choose_resident_shape(a2cid_ctx *c, const a2cid_event_batch *batch) {
    if (c->group != 0) {
        c->group_now = c->group;
        c->cols_now = c->resident_cols;
        return;
    }
    resident_shape(c->n, batch, &c->group_now, &c->cols_now);
}

static int apply_impl(a2cid_ctx *c, const a2cid_event_batch *batch) {
    if (int rc = enter(c)) return rc;
    if (int rc = unusable(c)) return rc;
    // ---- validation: nothing is enqueued and no time stamp moves before all of it has passed ----
    if (int rc = plan_batch(c->g, c->eta, c->t.data(), c->rate.data(), batch, c->plan, c->scratch)) return rc;
    // gradient inputs the kernels will read: d floats each, inside one device allocation
    c->known.clear();
    for (int64_t k = 0; k < batch->n_ops; ++k) {
        const a2cid_op &op = batch->ops[k];
        if (op.kind != A2CID_KIND_GRADIENT) continue;
        if (op.xi)
            if (int rc = check_device_span(c, op.xi, sizeof(float) * (size_t)c->d, "xi of a gradient event")) return rc;
        if (op.c && op.gscale != 0.f)
            if (int rc = check_device_span(c, op.c, sizeof(float) * (size_t)c->d, "c of a gradient event")) return rc;
        if (op.h && op.gscale != 0.f)
            if (int rc = check_device_span(c, op.h, sizeof(float) * (size_t)c->d, "h of a gradient event")) return rc;
    }
    const int64_t cap = piece_capacity(c);
    for (int32_t l = 0; l < batch->n_levels; ++l) {
        const int64_t sz = batch->level_off[l + 1] - batch->level_off[l];
        if (sz > cap) return fail(A2CID_EMATCHING, "level %d has %lld operations", l, (long long)sz);
    }
    // ---- enqueueing: a failure from here on leaves kernels in the stream whose time stamps were not committed ----
    if (int rc = enqueue_batch(c, batch)) {
        c->failed = true;
        return rc;
    }
    c->t = c->plan.t_after;
    c->rate = c->plan.rate_after;
    c->n_gossip += c->plan.n_gossip;
    c->n_grad += c->plan.n_grad;
    c->alg_bytes += (double)c->d * (32.0 * c->plan.n_gossip + 16.0 * c->plan.n_grad +
                                    4.0 * (c->plan.n_grad_xi + c->plan.n_grad_c + c->plan.n_grad_h));
    return A2CID_OK;
}

static int enqueue_batch(a2cid_ctx *c, const a2cid_event_batch *batch) {
    const int64_t cap = piece_capacity(c);
    const int mode = event_mode(c);
    if (mode == 2) {
        choose_resident_shape(c, batch);
        // as many launches as the programmes need (each holds resident_slots slots per wave)
        bool trailing = false;
        for (int64_t k = 0; k < batch->n_ops && !trailing; ++k)
            trailing = c->plan.coef[k].b_post_i != 0.f || c->plan.coef[k].b_post_j != 0.f;
        int32_t l = 0;
        int64_t k = 0;
        while (l < batch->n_levels) {
            if (k >= batch->level_off[l + 1]) { ++l; continue; }
            if (int rc = enqueue_resident(c, batch, &l, &k, trailing)) return rc;
        }
        return A2CID_OK;
    }
    if (mode == 4) {
        bool full = false, curvatures = false;
        for (int64_t q = 0; q < batch->n_ops && !curvatures; ++q) {
            const a2cid_op &op = batch->ops[q];
            if (op.kind != A2CID_KIND_GRADIENT || op.gscale == 0.f) continue;
            full = full || op.c || op.h;
            curvatures = op.h != nullptr;
        }
        int64_t k = 0;
        while (k < batch->n_ops)
            if (int rc = enqueue_regfile(c, batch, full, curvatures, &k)) return rc;
        return A2CID_OK;
    }
    int32_t l = 0;
    while (l < batch->n_levels) {
        // take as many whole levels as fit into one staging buffer (apply_impl has checked that every level does)
        int32_t l_end = l;
        int64_t count = 0;
        while (l_end < batch->n_levels) {
            const int64_t sz = batch->level_off[l_end + 1] - batch->level_off[l_end];
            if (sz > cap) return fail(A2CID_EMATCHING, "level %d has %lld operations", l_end, (long long)sz);
            if (count + sz > cap) break;
            count += sz;
            ++l_end;
        }
        if (count > 0) {
            Slot *s;
            if (int rc = acquire_slot(c, &s)) return rc;
            const int64_t first = batch->level_off[l];
            auto fill = [&](DevOp &o, int64_t src) {
                const a2cid_op &op = batch->ops[src];
                const a2cid_coef &cf = c->plan.coef[src];
                o.kind = (op.kind == A2CID_KIND_GOSSIP ? kOpGossip : kOpGradient) | (c->order ? kFlagListing << 8 : 0);
                o.row_i = op.i;
                o.row_j = op.kind == A2CID_KIND_GOSSIP ? op.j : op.i;
                o.b_i = cf.b_pre_i; o.b_j = cf.b_pre_j;
                o.bp_i = cf.b_post_i; o.bp_j = cf.b_post_j;
                o.gamma = op.gamma; o.gscale = op.gscale;
                o.xi = op.kind == A2CID_KIND_GRADIENT ? op.xi : nullptr;
                o.c = op.kind == A2CID_KIND_GRADIENT ? op.c : nullptr;
                o.h = op.kind == A2CID_KIND_GRADIENT ? op.h : nullptr;
                o.loc = 0;                  // every row from and to memory
            };
            int64_t n_dev = count;          // records of the device table
            if (mode == 3) {
                plan_chain(c->n, batch->ops + first, count, c->chain_slots, c->chain);
                n_dev = (int64_t)c->chain.steps.size();
                if (n_dev > kSlotOps) return fail(A2CID_EINVAL, "internal: chain programme of %lld steps", (long long)n_dev);
                for (int64_t k = 0; k < n_dev; ++k) {
                    const a2cid_chain_step &st = c->chain.steps[k];
                    DevOp &o = s->host[k];
                    const uint32_t top = kLocSlot0 + (uint32_t)c->chain_slots;
                    if (st.src_i >= top || st.src_j >= top || st.dst_i >= top || st.dst_j >= top)
                        return fail(A2CID_EINVAL, "internal: chain step %lld names a slot that does not exist", (long long)k);
                    if (st.op < 0) {
                        std::memset(&o, 0, sizeof(o));
                        o.kind = kOpSpill;
                        o.row_i = o.row_j = st.row_i;
                        o.loc = st.src_i;
                        continue;
                    }
                    fill(o, first + st.op);
                    if (o.row_i != st.row_i) {       // a gossip operation turned so that the carried worker is row_i
                        std::swap(o.row_i, o.row_j);
                        std::swap(o.b_i, o.b_j);
                        std::swap(o.bp_i, o.bp_j);
                    }
                    o.loc = (uint32_t)st.src_i | (uint32_t)st.src_j << 8 | (uint32_t)st.dst_i << 16 | (uint32_t)st.dst_j << 24;
                }
            } else {
                for (int64_t k = 0; k < count; ++k) fill(s->host[k], first + k);
            }
            double moved = 0.0;             // bytes per column that this chunk's launches move
            if (mode == 3) {
                moved = c->chain.bytes_per_column;
            } else {
                for (int64_t k = 0; k < count; ++k) {
                    const DevOp &o = s->host[k];
                    moved += op_kind(o.kind) == kOpGossip ? 32.0 : 16.0 + (o.xi ? 4.0 : 0.0) +
                             ((o.c && o.gscale != 0.f) ? 4.0 : 0.0) + ((o.h && o.gscale != 0.f) ? 4.0 : 0.0);
                }
            }
            c->moved_bytes += moved * (double)c->d;
            A2CID_HIP(hipMemcpyAsync(s->dev, s->host, sizeof(DevOp) * (size_t)n_dev, hipMemcpyHostToDevice, c->stream));
            if (mode == 3) {
                if (int rc = launch_ops(c, s->dev, (int32_t)n_dev, kLaunchChain)) return rc;
            } else if (mode == 1) {
                if (int rc = launch_ops(c, s->dev, (int32_t)count, kLaunchWalk)) return rc;
            } else {
                for (int32_t ll = l; ll < l_end; ++ll) {
                    const int64_t lo = batch->level_off[ll] - first, sz = batch->level_off[ll + 1] - batch->level_off[ll];
                    if (sz == 0) continue;
                    if (int rc = launch_ops(c, s->dev + lo, (int32_t)sz, kLaunchLevel)) return rc;
                }
            }
            A2CID_HIP(hipEventRecord(s->done, c->stream));
            s->in_flight = true;
        }
        l = l_end;
    }
    return A2CID_OK;
}

int a2cid_apply_events(a2cid_ctx *c, const a2cid_event_batch *batch) {
    clear_error();
    if (!c) return fail(A2CID_EINVAL, "context is NULL");
    try {
        return apply_impl(c, batch);
    } catch (const std::bad_alloc &) {
        return fail(A2CID_ENOMEM, "out of host memory");
    }
}

// Checks shared by the calls that bring every worker to a common time t_now.
static int check_common_time(const a2cid_ctx *c, double t_now) {
    if (!std::isfinite(t_now)) return fail(A2CID_EINVAL, "t_now is not finite");
    if (int rc = enter(c)) return rc;
    if (int rc = unusable(c)) return rc;
    for (int32_t i = 0; i < c->n; ++i)
        if (t_now < c->t[i]) return fail(A2CID_EORDER, "t_now %.17g is before worker %d's time %.17g", t_now, i, c->t[i]);
    return A2CID_OK;
}

// Uploads the n pending mixing coefficients for t_now into b_dev (stream-ordered after every earlier reader of it).
static int upload_coefficients(a2cid_ctx *c, double t_now) {
    CoefStage *cs;
    if (int rc = acquire_coef_stage(c, &cs)) return rc;
    for (int32_t i = 0; i < c->n; ++i) cs->host[i] = (float)mix_coefficient(c->eta, c->rate[i] * (t_now - c->t[i]));
    A2CID_HIP(hipMemcpyAsync(c->b_dev, cs->host, sizeof(float) * c->n, hipMemcpyHostToDevice, c->stream));
    A2CID_HIP(hipEventRecord(cs->done, c->stream));
    cs->in_flight = true;
    return A2CID_OK;
}

int a2cid_flush(a2cid_ctx *c, double t_now) {
    clear_error();
    if (!c) return fail(A2CID_EINVAL, "context is NULL");
    if (int rc = check_common_time(c, t_now)) return rc;
    try {
        std::vector<float> b(c->n);
        for (int32_t i = 0; i < c->n; ++i) b[i] = (float)mix_coefficient(c->eta, c->rate[i] * (t_now - c->t[i]));
        if (int rc = enqueue_mix_all(c, b)) {
            c->failed = true;
            return rc;
        }
    } catch (const std::bad_alloc &) {
        return fail(A2CID_ENOMEM, "out of host memory");
    }
    std::fill(c->t.begin(), c->t.end(), t_now);
    return A2CID_OK;
}

// The observables pass: per-workgroup partials into `partials` (blocks x (2n + 2) doubles), then their sums into
// `out` (2n + 2 doubles: sums of x, sums of xt, the two consensus distances).  The coefficients come from the
// device table b_dev, or, when args is not NULL, from the kernel's argument block.
static int launch_stats(a2cid_ctx *c, const float *b_dev, const MixArgs *args, double *partials, int32_t max_blocks,
                        double *out) {
    const int64_t pieces = (c->d + 3) >> 2;
    const int v = c->stats_v, r = c->stats_r;
    const int64_t per_tile = (int64_t)v * kThreads;
    const int64_t n_tiles = (pieces + per_tile - 1) / per_tile;
    const int32_t blocks = (int32_t)std::min<int64_t>(n_tiles, max_blocks);
    const int32_t m = 2 * c->n + 2;
    const size_t lds = sizeof(double) * kWaves * 2 * (size_t)c->n + sizeof(float) * (size_t)c->n;
    // timing is a measurement aid of the allocating entry point only: a2cid_stats_static (args != NULL) takes no events
    TimedLaunch tl{};
    const bool timing = c->profiling && !args;
    if (timing) {
        if (int rc = get_event(c, &tl.start)) return rc;
        if (int rc = get_event(c, &tl.stop)) return rc;
        A2CID_HIP(hipEventRecord(tl.start, c->stream));
    }
#define A2CID_STATS_LAUNCH(V, R, NT)                                                                             \
    do {                                                                                                         \
        if (args) {      /* at most kMixArgsMax workers: the dynamic LDS stays below the default cap */            \
            hipLaunchKernelGGL((stats_args_kernel<V, R, NT>), dim3(blocks), dim3(kThreads), lds, c->stream, c->x, \
                               c->xt, c->ld, c->d, c->n, *args, partials, n_tiles);                               \
        } else {                                                                                                 \
            if (lds > 32768)   /* the kernel also has 4 KiB of static LDS; the default cap is 64 KiB in total */  \
                A2CID_HIP(hipFuncSetAttribute((const void *)stats_kernel<V, R, NT>,                               \
                                              hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));             \
            hipLaunchKernelGGL((stats_kernel<V, R, NT>), dim3(blocks), dim3(kThreads), lds, c->stream, c->x,      \
                               c->xt, c->ld, c->d, c->n, b_dev, partials, n_tiles);                               \
        }                                                                                                        \
    } while (0)
    const bool snt = c->stats_nt != 0;
    if (v == 1 && r == 1) { if (snt) A2CID_STATS_LAUNCH(1, 1, true); else A2CID_STATS_LAUNCH(1, 1, false); }
    else if (v == 1 && r == 2) { if (snt) A2CID_STATS_LAUNCH(1, 2, true); else A2CID_STATS_LAUNCH(1, 2, false); }
    else if (v == 1 && r == 4) { if (snt) A2CID_STATS_LAUNCH(1, 4, true); else A2CID_STATS_LAUNCH(1, 4, false); }
    else if (v == 2 && r == 1) { if (snt) A2CID_STATS_LAUNCH(2, 1, true); else A2CID_STATS_LAUNCH(2, 1, false); }
    else if (v == 2 && r == 4) { if (snt) A2CID_STATS_LAUNCH(2, 4, true); else A2CID_STATS_LAUNCH(2, 4, false); }
    else { if (snt) A2CID_STATS_LAUNCH(2, 2, true); else A2CID_STATS_LAUNCH(2, 2, false); }
#undef A2CID_STATS_LAUNCH
    A2CID_HIP(hipGetLastError());
    if (timing) {
        A2CID_HIP(hipEventRecord(tl.stop, c->stream));
        c->timed_stats.push_back(tl);
    }
    hipLaunchKernelGGL(stats_final_kernel, dim3(m), dim3(kThreads), 0, c->stream, partials, blocks, m, out);
    A2CID_HIP(hipGetLastError());
    return A2CID_OK;
}

static int stats_impl(a2cid_ctx *c, double t_now) {
    if (int rc = upload_coefficients(c, t_now)) return rc;
    if (int rc = launch_stats(c, c->b_dev, nullptr, c->partials, c->stats_blocks, c->out_dev)) return rc;
    const int32_t m = 2 * c->n + 2;
    A2CID_HIP(hipMemcpyAsync(c->out_host, c->out_dev, sizeof(double) * m, hipMemcpyDeviceToHost, c->stream));
    A2CID_HIP(hipStreamSynchronize(c->stream));
    return A2CID_OK;
}

int a2cid_stats(a2cid_ctx *c, double t_now, a2cid_stats_out *out) {
    clear_error();
    if (!c || !out || !out->sum_x || !out->sum_xt) return fail(A2CID_EINVAL, "context / out is NULL");
    if (int rc = check_common_time(c, t_now)) return rc;
    if (int rc = stats_impl(c, t_now)) {
        c->failed = true;
        return rc;
    }
    std::memcpy(out->sum_x, c->out_host, sizeof(double) * c->n);
    std::memcpy(out->sum_xt, c->out_host + c->n, sizeof(double) * c->n);
    out->consensus_x = c->out_host[2 * c->n];
    out->consensus_xt = c->out_host[2 * c->n + 1];
    return A2CID_OK;
}

int a2cid_stats_static(a2cid_ctx *c, double t_now, double *out) {
    clear_error();
    if (!c || !out) return fail(A2CID_EINVAL, "context / out is NULL");
    if (c->n > A2CID_STATS_STATIC_MAX_WORKERS)
        return fail(A2CID_EINVAL, "a2cid_stats_static handles at most %d workers (the context has %d): its scratch is "
                    "a fixed array of %zu bytes and its coefficients travel in the kernel arguments",
                    A2CID_STATS_STATIC_MAX_WORKERS, c->n, sizeof(double) * kStaticDoubles);
    if ((uintptr_t)out & 7u) return fail(A2CID_EALIGN, "out must be 8-byte aligned");
    if (int rc = check_common_time(c, t_now)) return rc;
    const int32_t m = 2 * c->n + 2;
    if (int rc = query_device_span(c, out, sizeof(double) * (size_t)m, "out", nullptr)) return rc;
    double *partials = nullptr;
    if (int rc = static_scratch(c->device, &partials)) return rc;
    MixArgs args;
    for (int32_t i = 0; i < kMixArgsMax; ++i)
        args.b[i] = i < c->n ? (float)mix_coefficient(c->eta, c->rate[i] * (t_now - c->t[i])) : 0.f;
    const int32_t max_blocks = (int32_t)std::min<size_t>((size_t)c->stats_blocks, kStaticDoubles / (size_t)m);
    if (int rc = launch_stats(c, nullptr, &args, partials, max_blocks, out)) {
        c->failed = true;
        return rc;
    }
    return A2CID_OK;
}

static int average_impl(a2cid_ctx *c, double t_now) {
    if (int rc = upload_coefficients(c, t_now)) return rc;
    const int64_t pieces = (c->d + 3) >> 2;
    hipLaunchKernelGGL(average_kernel, dim3((unsigned)((pieces + kThreads - 1) / kThreads)), dim3(kThreads),
                       sizeof(float) * (size_t)c->n, c->stream, c->x, c->xt, c->ld, c->d, c->n, c->b_dev);
    A2CID_HIP(hipGetLastError());
    return A2CID_OK;
}

int a2cid_average(a2cid_ctx *c, double t_now) {
    clear_error();
    if (!c) return fail(A2CID_EINVAL, "context is NULL");
    if (int rc = check_common_time(c, t_now)) return rc;
    if (int rc = average_impl(c, t_now)) {
        c->failed = true;
        return rc;
    }
    std::fill(c->t.begin(), c->t.end(), t_now);
    c->alg_bytes += 16.0 * (double)c->n * (double)c->d;
    c->moved_bytes += 16.0 * (double)c->n * (double)c->d;
    return A2CID_OK;
}

int a2cid_get_times(const a2cid_ctx *c, double *t) {
    clear_error();
    if (!c || !t) return fail(A2CID_EINVAL, "context / t is NULL");
    std::copy(c->t.begin(), c->t.end(), t);
    return A2CID_OK;
}

int a2cid_get_clock_rates(const a2cid_ctx *c, double *rate) {
    clear_error();
    if (!c || !rate) return fail(A2CID_EINVAL, "context / rate is NULL");
    std::copy(c->rate.begin(), c->rate.end(), rate);
    return A2CID_OK;
}

int a2cid_set_clock_rates(a2cid_ctx *c, const double *rate) {
    clear_error();
    if (!c || !rate) return fail(A2CID_EINVAL, "context / rate is NULL");
    for (int32_t i = 0; i < c->n; ++i)
        if (!(rate[i] > 0.0) || !std::isfinite(rate[i])) return fail(A2CID_EINVAL, "rate[%d] must be finite and > 0", i);
    c->rate.assign(rate, rate + c->n);
    return A2CID_OK;
}

int a2cid_set_times(a2cid_ctx *c, const double *t) {
    clear_error();
    if (!c || !t) return fail(A2CID_EINVAL, "context / t is NULL");
    for (int32_t i = 0; i < c->n; ++i)
        if (!std::isfinite(t[i])) return fail(A2CID_EINVAL, "t[%d] is not finite", i);
    c->t.assign(t, t + c->n);
    return A2CID_OK;
}

int a2cid_synchronize(a2cid_ctx *c) {
    clear_error();
    if (!c) return fail(A2CID_EINVAL, "context is NULL");
    A2CID_HIP(hipStreamSynchronize(c->stream));
    return A2CID_OK;
}

int a2cid_set_tuning(a2cid_ctx *c, int32_t unroll, int32_t nontemporal, int32_t threads, int32_t mode) {
    clear_error();
    if (!c) return fail(A2CID_EINVAL, "context is NULL");
    if (unroll != 1 && unroll != 2 && unroll != 4) return fail(A2CID_EINVAL, "unroll must be 1, 2 or 4");
    if (threads != 64 && threads != 128 && threads != 256 && threads != 512 && threads != 1024)
        return fail(A2CID_EINVAL, "threads must be 64, 128, 256, 512 or 1024");
    if (mode < -1 || mode > 4)
        return fail(A2CID_EINVAL, "mode must be -1 (automatic), 0 (levels), 1 (walk), 2 (resident), 3 (chain) or 4 (register file)");
    if (mode == 4 && (c->n > kRegMaxRows || c->d > kRegMaxColumns))
        return fail(A2CID_EINVAL, "the register-file kernel holds at most %d workers of at most 2^29 parameters", kRegMaxRows);
    if (mode == 2 && c->n > kResidentMaxRows)
        return fail(A2CID_EINVAL, "the resident kernel holds at most %d workers in LDS", kResidentMaxRows);
    if ((mode == 3 || mode == -1) && (size_t)c->chain_slots * unroll * threads * 32 > 160 * 1024)
        return fail(A2CID_EINVAL, "%d slots of %d x %d lanes x 32 bytes do not fit into 160 KiB of LDS "
                    "(a2cid_set_chain_slots lowers the slots)", c->chain_slots, unroll, threads);
    c->unroll = unroll;
    c->nontemporal = nontemporal ? 1 : 0;
    c->threads = threads;
    c->walk = mode;
    return A2CID_OK;
}

int a2cid_set_order(a2cid_ctx *c, int32_t order) {
    clear_error();
    if (!c) return fail(A2CID_EINVAL, "context is NULL");
    if (order != A2CID_ORDER_EQ1 && order != A2CID_ORDER_LISTING) return fail(A2CID_EINVAL, "unknown order %d", order);
    c->order = order;
    return A2CID_OK;
}

int a2cid_set_chain_slots(a2cid_ctx *c, int32_t slots) {
    clear_error();
    if (!c) return fail(A2CID_EINVAL, "context is NULL");
    if (slots < 0 || slots > kChainMaxSlots) return fail(A2CID_EINVAL, "slots must be in [0, %d]", kChainMaxSlots);
    if ((size_t)slots * c->unroll * c->threads * 32 > 160 * 1024)
        return fail(A2CID_EINVAL, "%d slots of %d x %d lanes x 32 bytes do not fit into 160 KiB of LDS", slots, c->unroll,
                    c->threads);
    c->chain_slots = slots;
    return A2CID_OK;
}

int a2cid_set_walk_occupancy(a2cid_ctx *c, int32_t workgroups_per_cu) {
    clear_error();
    if (!c) return fail(A2CID_EINVAL, "context is NULL");
    if (workgroups_per_cu < 0 || workgroups_per_cu > 32) return fail(A2CID_EINVAL, "workgroups_per_cu must be in [0, 32]");
    c->walk_wg_per_cu = workgroups_per_cu;
    return A2CID_OK;
}

int a2cid_set_resident_group(a2cid_ctx *c, int32_t group, int32_t cols) {
    clear_error();
    if (!c) return fail(A2CID_EINVAL, "context is NULL");
    if (group == 0) {                   // back to the choice per batch
        c->group = 0;
        return A2CID_OK;
    }
    if (group != 1 && group != 2 && group != 4 && group != 8 && group != 16)
        return fail(A2CID_EINVAL, "group must be 0 (chosen per batch), 1, 2, 4, 8 or 16");
    if (cols != 1 && cols != 2 && cols != 4) return fail(A2CID_EINVAL, "cols must be 1, 2 or 4");
    if (group == 1 && cols != 1) return fail(A2CID_EINVAL, "group = 1 goes with cols = 1 only");
    if (resident_lds_bytes(cols, c->n) > 160 * 1024)
        return fail(A2CID_EINVAL, "%d workers x %d columns per lane do not fit into 160 KiB of LDS", c->n, cols);
    c->group = group;
    c->resident_cols = cols;
    return A2CID_OK;
}

int a2cid_set_stats_tuning(a2cid_ctx *c, int32_t pieces, int32_t rows, int32_t blocks, int32_t nontemporal) {
    clear_error();
    if (!c) return fail(A2CID_EINVAL, "context is NULL");
    if ((pieces != 1 && pieces != 2) || (rows != 1 && rows != 2 && rows != 4))
        return fail(A2CID_EINVAL, "pieces must be 1 or 2 and rows 1, 2 or 4");
    if (blocks < 1 || blocks > kStatsBlocksMax) return fail(A2CID_EINVAL, "blocks must be in [1, %d]", kStatsBlocksMax);
    c->stats_v = pieces; c->stats_r = rows; c->stats_blocks = blocks; c->stats_nt = nontemporal ? 1 : 0;
    return A2CID_OK;
}

int a2cid_check_device_span(a2cid_ctx *c, const void *p, int64_t bytes) {
    clear_error();
    if (!c || !p || bytes < 1) return fail(A2CID_EINVAL, "context / pointer NULL or bytes < 1");
    return query_device_span(c, p, (size_t)bytes, "span", nullptr);
}

int a2cid_stream_probe(const float *src, float *dst, int64_t n, void *hip_stream) {
    clear_error();
    if (!src || !dst || n < 4 || (n & 3)) return fail(A2CID_EINVAL, "src / dst NULL or n not a positive multiple of 4");
    if (((uintptr_t)src | (uintptr_t)dst) & 15u) return fail(A2CID_EALIGN, "src and dst must be 16-byte aligned");
    const int64_t n4 = n >> 2;
    hipLaunchKernelGGL(copy_probe_kernel, dim3((unsigned)((n4 + 1023) / 1024)), dim3(256), 0, (hipStream_t)hip_stream,
                       (const v4f *)src, (v4f *)dst, n4);
    A2CID_HIP(hipGetLastError());
    return A2CID_OK;
}

int a2cid_counters(a2cid_ctx *c, int64_t *n_gossip, int64_t *n_gradient, int64_t *n_launches,
                   double *one_pass_bytes, double *moved_bytes, int32_t reset) {
    clear_error();
    if (!c) return fail(A2CID_EINVAL, "context is NULL");
    if (n_gossip) *n_gossip = c->n_gossip;
    if (n_gradient) *n_gradient = c->n_grad;
    if (n_launches) *n_launches = c->n_launch;
    if (one_pass_bytes) *one_pass_bytes = c->alg_bytes;
    if (moved_bytes) *moved_bytes = c->moved_bytes;
    if (reset) { c->n_gossip = c->n_grad = c->n_launch = 0; c->alg_bytes = c->moved_bytes = 0.0; }
    return A2CID_OK;
}

int a2cid_profile(a2cid_ctx *c, int32_t enable) {
    clear_error();
    if (!c) return fail(A2CID_EINVAL, "context is NULL");
    c->profiling = enable != 0;
    return A2CID_OK;
}

static int read_timed(a2cid_ctx *c, std::vector<TimedLaunch> &timed, int64_t *n_launches, double *kernel_ms) {
    A2CID_HIP(hipStreamSynchronize(c->stream));
    double total = 0.0;
    for (TimedLaunch &tl : timed) {
        float ms = 0.f;
        A2CID_HIP(hipEventElapsedTime(&ms, tl.start, tl.stop));
        total += ms;
        c->event_pool.push_back(tl.start);
        c->event_pool.push_back(tl.stop);
    }
    if (n_launches) *n_launches = (int64_t)timed.size();
    if (kernel_ms) *kernel_ms = total;
    timed.clear();
    return A2CID_OK;
}

int a2cid_profile_read(a2cid_ctx *c, int64_t *n_launches, double *kernel_ms) {
    clear_error();
    if (!c) return fail(A2CID_EINVAL, "context is NULL");
    return read_timed(c, c->timed, n_launches, kernel_ms);
}

int a2cid_profile_read_stats(a2cid_ctx *c, int64_t *n_launches, double *kernel_ms) {
    clear_error();
    if (!c) return fail(A2CID_EINVAL, "context is NULL");
    return read_timed(c, c->timed_stats, n_launches, kernel_ms);
}

int a2cid_inplace_probe(a2cid_ctx *c, int32_t rows_per_op, int32_t n_ops, double *bytes) {
    clear_error();
    if (!c) return fail(A2CID_EINVAL, "context is NULL");
    if (rows_per_op != 1 && rows_per_op != 2) return fail(A2CID_EINVAL, "rows_per_op must be 1 or 2");
    if (n_ops < 1) return fail(A2CID_EINVAL, "n_ops must be >= 1");
    if (int rc = enter(c)) return rc;
    if (int rc = unusable(c)) return rc;
    const int64_t n4 = c->d >> 2;
    if (bytes) *bytes = (double)n_ops * rows_per_op * 64.0 * (double)n4;
    if (n4 == 0) return A2CID_OK;
    const dim3 grid((unsigned)((n4 + kThreads - 1) / kThreads)), block(kThreads);
    if (rows_per_op == 2)
        hipLaunchKernelGGL((inplace_probe_kernel<2, kThreads>), grid, block, 0, c->stream, c->x, c->xt, c->ld, c->d, c->n,
                           n_ops, 1.0f);
    else
        hipLaunchKernelGGL((inplace_probe_kernel<1, kThreads>), grid, block, 0, c->stream, c->x, c->xt, c->ld, c->d, c->n,
                           n_ops, 1.0f);
    A2CID_HIP(hipGetLastError());
    return A2CID_OK;
}

}  // extern "C"
