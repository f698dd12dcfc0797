// Device code of the A2CiD2 engine for gfx950 (wave64).  Included only by a2cid_engine.hip.
//
// The event kernels (level, walk) and the observables kernel are HBM streams (about 0.5 flop per
// byte), so there is no MFMA and no LDS on their data path: each lane moves 128-bit pieces straight
// between global memory and registers, and the design goal is simply "enough independent 16-byte
// loads in flight per CU".  The resident kernel is the exception: it keeps a column tile of
// every touched row in LDS for the length of a batch.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace a2cid {

typedef float v4f __attribute__((ext_vector_type(4)));

constexpr int kThreads = 256;           // 4 wavefronts per workgroup
constexpr int kWaves = kThreads / 64;

enum : int32_t { kOpGradient = 0, kOpGossip = 1, kOpMixOnly = 2, kOpSpill = 3 };

// One operation of a level as the kernels see it (64 bytes).  Every field is uniform across
// the workgroup that executes the operation, so the compiler keeps it in scalar registers.
struct DevOp {
    int32_t kind;                // kOp* in the low byte, kFlag* bits above it (op_kind, op_flags)
    int32_t row_i, row_j;        // worker rows (row_j unused unless gossip)
    float b_i, b_j;              // mixing to the event time: off-diagonal of exp(tau A)
    float bp_i, bp_j;            // trailing mixing (0 = none)
    float gamma, gscale;         // gradient step size and slope of the affine gradient model
    uint32_t loc;                // chain kernel: where the rows come from and go to, one kLoc* code per byte:
                                 // src_i | src_j << 8 | dst_i << 16 | dst_j << 24 (32-bit fields only: the
                                 // record then stays in scalar registers)
    const float *xi;             // additive gradient term or nullptr
    const float *c;              // centre of the affine gradient model or nullptr
    const float *h;              // per-coordinate curvature of the gradient model or nullptr (ones)
};
static_assert(sizeof(DevOp) == 64, "DevOp layout");

enum : int32_t {
    kFlagListing = 1,            // jumps from the stored (pre-mix) values, Algorithm 1's listing order
};
__host__ __device__ __forceinline__ int32_t op_kind(int32_t word) { return word & 255; }
__host__ __device__ __forceinline__ int32_t op_flags(int32_t word) { return word >> 8; }

// Chain kernel: where a worker's columns of the workgroup's tile are.
enum : uint32_t {
    kLocMemory = 0,              // the row in device memory
    kLocCarry = 1,               // the workgroup's carry registers (from one operation to the very next)
    kLocSlot0 = 2,               // kLocSlot0 + s: parked in LDS slot s
};

// The arithmetic of the three updates is written with explicit fused multiply-adds, so that every kernel performs
// the same sequence of individually rounded IEEE operations whatever the compiler would have chosen to contract in
// its context: this is what makes the kernels agree bit for bit.
__device__ __forceinline__ float fma_s(float s, float a, float c) { return __builtin_fmaf(s, a, c); }
__device__ __forceinline__ v4f fma_s(float s, v4f a, v4f c) {
    const v4f sv = {s, s, s, s};
    return __builtin_elementwise_fma(sv, a, c);
}
__device__ __forceinline__ float fma_t(float s, float a, float c) { return __builtin_fmaf(s, a, c); }
__device__ __forceinline__ v4f fma_t(v4f s, v4f a, v4f c) { return __builtin_elementwise_fma(s, a, c); }

// exp(tau A) (x, xt) in increment form: with b the off-diagonal entry and delta = xt - x, x <- x + b delta and
// xt <- xt - b delta (one rounding each).  x + xt is conserved up to rounding; b = 0 is the identity.
template <typename T>
__device__ __forceinline__ void mix(T &x, T &xt, float b) {
    const T delta = xt - x;
    x = fma_s(b, delta, x);
    xt = fma_s(-b, delta, xt);
}

// Gossip jump of Eq. (1) for one pair, including the flows before and (optionally) after it.
// pre = false: the difference m is taken after both workers are mixed (Eq. (1));
// pre = true:  m is taken from the stored values, before the mixing (Algorithm 1 as listed).
template <typename T, typename Op>
__device__ __forceinline__ void gossip_update(T &xi, T &xti, T &xj, T &xtj, const Op &op,
                                              float alpha, float alpha_t, bool pre) {
    const T m_stored = xi - xj;
    mix(xi, xti, op.b_i);
    mix(xj, xtj, op.b_j);
    const T m = pre ? m_stored : xi - xj;
    xi = fma_s(-alpha, m, xi);
    xj = fma_s(alpha, m, xj);
    xti = fma_s(-alpha_t, m, xti);
    xtj = fma_s(alpha_t, m, xtj);
    mix(xi, xti, op.bp_i);
    mix(xj, xtj, op.bp_j);
}

// Gradient jump of Eq. (1) with g = gscale h (x - c) + xi (h: the coordinate's curvature, 1 when the event
// carries none: gscale * 1 is exact), taken at the mixed point (pre = false) or at the stored point (pre = true,
// Algorithm 1 as listed).
template <typename T, typename Op>
__device__ __forceinline__ void gradient_update(T &x, T &xt, T xi, T c, T h, const Op &op, bool pre) {
    const T slope = op.gscale * h;
    const T g_stored = fma_t(slope, x - c, xi);
    mix(x, xt, op.b_i);
    const T g = pre ? g_stored : fma_t(slope, x - c, xi);
    x = fma_s(-op.gamma, g, x);
    xt = fma_s(-op.gamma, g, xt);
    mix(x, xt, op.bp_i);
}

// The same two jumps with the trailing mix as a compile-time case: a mix with b = 0 is the identity (the fused
// multiply-add of 0 * delta onto x returns x; only a negative zero would come back positive), so without a trailing
// mix its instructions are simply left out.
template <bool TRAIL, typename T, typename Op>
__device__ __forceinline__ void gossip_jump(T &xi, T &xti, T &xj, T &xtj, const Op &op, float alpha, float alpha_t,
                                            bool pre) {
    const T m_stored = xi - xj;
    mix(xi, xti, op.b_i);
    mix(xj, xtj, op.b_j);
    const T m = pre ? m_stored : xi - xj;
    xi = fma_s(-alpha, m, xi);
    xj = fma_s(alpha, m, xj);
    xti = fma_s(-alpha_t, m, xti);
    xtj = fma_s(alpha_t, m, xtj);
    if (TRAIL) { mix(xi, xti, op.bp_i); mix(xj, xtj, op.bp_j); }
}

template <bool TRAIL, typename T, typename Op>
__device__ __forceinline__ void gradient_jump(T &x, T &xt, T xi, T c, T h, const Op &op, bool pre) {
    const T slope = op.gscale * h;
    const T g_stored = fma_t(slope, x - c, xi);
    mix(x, xt, op.b_i);
    const T g = pre ? g_stored : fma_t(slope, x - c, xi);
    x = fma_s(-op.gamma, g, x);
    xt = fma_s(-op.gamma, g, xt);
    if (TRAIL) mix(x, xt, op.bp_i);
}

template <bool NT>
__device__ __forceinline__ v4f load4(const v4f *p) {
    if constexpr (NT) return __builtin_nontemporal_load(p);
    else return *p;
}
template <bool NT>
__device__ __forceinline__ void store4(v4f *p, v4f v) {
    if constexpr (NT) __builtin_nontemporal_store(v, p);
    else *p = v;
}

// ------------------------------------------------------------------------------------------
// One operation applied to one tile of U * TPB float4 columns by a workgroup of TPB lanes:
// every lane loads U 16-byte pieces of each row the operation touches (coalesced: consecutive
// lanes, consecutive 16 bytes), updates them in registers and stores them back in place.
//   gossip:   4 rows in, 4 rows out  (32 bytes per column)
//   gradient: 2 rows (+ xi, + c) in, 2 rows out  (16 / 20 / 24 bytes per column)
//   mix only: 2 rows in, 2 rows out
// Gradient inputs are read once and never written, so their loads are always non-temporal: kept out
// of the caches they leave more room for state lines (measured +5 % on the ring workload, where a
// third of the events are gradient events; neutral elsewhere).  For the state rows NT selects the policy.
// The d % 4 trailing columns of a row are handled by scalar code in tile 0.
// ------------------------------------------------------------------------------------------
template <int U, bool NT, int TPB>
__device__ __forceinline__ void apply_op_tile(float *__restrict__ x, float *__restrict__ xt, int64_t ld,
                                              int64_t d, const DevOp &op, int64_t tile,
                                              float alpha, float alpha_t) {
    const int64_t n4 = d >> 2;                                   // whole float4 pieces per row
    const bool pre = (op_flags(op.kind) & kFlagListing) != 0;
    const int32_t kind = op_kind(op.kind);
    const int64_t base = (int64_t)tile * (U * TPB) + threadIdx.x;
    const bool full = (int64_t)(tile + 1) * (U * TPB) <= n4;

    float *xi_row = x + (int64_t)op.row_i * ld;
    float *xti_row = xt + (int64_t)op.row_i * ld;

    if (kind == kOpGossip) {
        float *xj_row = x + (int64_t)op.row_j * ld;
        float *xtj_row = xt + (int64_t)op.row_j * ld;
        v4f *pi = (v4f *)xi_row, *pti = (v4f *)xti_row, *pj = (v4f *)xj_row, *ptj = (v4f *)xtj_row;
        v4f a[U], at[U], b[U], bt[U];
        if (full) {
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int64_t k = base + u * TPB;
                a[u] = load4<NT>(pi + k); at[u] = load4<NT>(pti + k);
                b[u] = load4<NT>(pj + k); bt[u] = load4<NT>(ptj + k);
            }
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int64_t k = base + u * TPB;
                gossip_update(a[u], at[u], b[u], bt[u], op, alpha, alpha_t, pre);
                store4<NT>(pi + k, a[u]); store4<NT>(pti + k, at[u]);
                store4<NT>(pj + k, b[u]); store4<NT>(ptj + k, bt[u]);
            }
        } else {
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int64_t k = base + u * TPB;
                if (k < n4) {
                    a[u] = pi[k]; at[u] = pti[k]; b[u] = pj[k]; bt[u] = ptj[k];
                    gossip_update(a[u], at[u], b[u], bt[u], op, alpha, alpha_t, pre);
                    pi[k] = a[u]; pti[k] = at[u]; pj[k] = b[u]; ptj[k] = bt[u];
                }
            }
        }
        if (tile == 0) {
            const int64_t k = (n4 << 2) + threadIdx.x;
            if (threadIdx.x < 4 && k < d) {
                float s0 = xi_row[k], s1 = xti_row[k], s2 = xj_row[k], s3 = xtj_row[k];
                gossip_update(s0, s1, s2, s3, op, alpha, alpha_t, pre);
                xi_row[k] = s0; xti_row[k] = s1; xj_row[k] = s2; xtj_row[k] = s3;
            }
        }
    } else {
        v4f *pi = (v4f *)xi_row, *pti = (v4f *)xti_row;
        const bool grad = kind == kOpGradient;
        const bool has_xi = grad && op.xi != nullptr;
        const bool has_c = grad && op.c != nullptr && op.gscale != 0.f;
        const bool has_h = grad && op.h != nullptr && op.gscale != 0.f;
        const v4f *pxi = (const v4f *)op.xi, *pc = (const v4f *)op.c, *ph = (const v4f *)op.h;
        const v4f zero = {0.f, 0.f, 0.f, 0.f}, one = {1.f, 1.f, 1.f, 1.f};
        v4f a[U], at[U], g[U], c[U], h[U];
        if (full) {
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int64_t k = base + u * TPB;
                a[u] = load4<NT>(pi + k); at[u] = load4<NT>(pti + k);
                g[u] = has_xi ? load4<true>(pxi + k) : zero;
                c[u] = has_c ? load4<true>(pc + k) : zero;
                h[u] = has_h ? load4<true>(ph + k) : one;
            }
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int64_t k = base + u * TPB;
                if (grad) gradient_update(a[u], at[u], g[u], c[u], h[u], op, pre);
                else mix(a[u], at[u], op.b_i);
                store4<NT>(pi + k, a[u]); store4<NT>(pti + k, at[u]);
            }
        } else {
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int64_t k = base + u * TPB;
                if (k < n4) {
                    a[u] = pi[k]; at[u] = pti[k];
                    g[u] = has_xi ? pxi[k] : zero;
                    c[u] = has_c ? pc[k] : zero;
                    h[u] = has_h ? ph[k] : one;
                    if (grad) gradient_update(a[u], at[u], g[u], c[u], h[u], op, pre);
                    else mix(a[u], at[u], op.b_i);
                    pi[k] = a[u]; pti[k] = at[u];
                }
            }
        }
        if (tile == 0) {
            const int64_t k = (n4 << 2) + threadIdx.x;
            if (threadIdx.x < 4 && k < d) {
                float s0 = xi_row[k], s1 = xti_row[k];
                const float gk = has_xi ? op.xi[k] : 0.f, ck = has_c ? op.c[k] : 0.f, hk = has_h ? op.h[k] : 1.f;
                if (grad) gradient_update(s0, s1, gk, ck, hk, op, pre);
                else mix(s0, s1, op.b_i);
                xi_row[k] = s0; xti_row[k] = s1;
            }
        }
    }
}

// ------------------------------------------------------------------------------------------
// Level kernel: grid = (column tiles, operations of one level); one launch per level.
// Operations of a level touch disjoint rows, so no two workgroups of a launch ever touch the
// same byte, and the launch boundary orders consecutive levels.
// ------------------------------------------------------------------------------------------
template <int U, bool NT, int TPB>
__global__ __launch_bounds__(TPB) void level_kernel(float *__restrict__ x, float *__restrict__ xt,
                                                    int64_t ld, int64_t d, const DevOp *__restrict__ ops,
                                                    float alpha, float alpha_t) {
    const DevOp op = ops[blockIdx.y];
    apply_op_tile<U, NT, TPB>(x, xt, ld, d, op, (int64_t)blockIdx.x, alpha, alpha_t);
}

// The d % 4 trailing columns of the rows of one operation, by lanes 0..3 of the calling workgroup, always
// through memory (no carry).
__device__ __forceinline__ void apply_op_tail(float *__restrict__ x, float *__restrict__ xt, int64_t ld, int64_t d,
                                              const DevOp &op, float alpha, float alpha_t) {
    const int64_t k = ((d >> 2) << 2) + threadIdx.x;
    const int32_t kind = op_kind(op.kind);
    if (threadIdx.x >= 4 || k >= d || kind == kOpSpill) return;
    const bool pre = (op_flags(op.kind) & kFlagListing) != 0;
    float *xi_row = x + (int64_t)op.row_i * ld, *xti_row = xt + (int64_t)op.row_i * ld;
    float s0 = xi_row[k], s1 = xti_row[k];
    if (kind == kOpGossip) {
        float *xj_row = x + (int64_t)op.row_j * ld, *xtj_row = xt + (int64_t)op.row_j * ld;
        float s2 = xj_row[k], s3 = xtj_row[k];
        gossip_update(s0, s1, s2, s3, op, alpha, alpha_t, pre);
        xj_row[k] = s2; xtj_row[k] = s3;
    } else if (kind == kOpGradient) {
        const float gk = op.xi != nullptr ? op.xi[k] : 0.f;
        const float ck = (op.c != nullptr && op.gscale != 0.f) ? op.c[k] : 0.f;
        const float hk = (op.h != nullptr && op.gscale != 0.f) ? op.h[k] : 1.f;
        gradient_update(s0, s1, gk, ck, hk, op, pre);
    } else {
        mix(s0, s1, op.b_i);
    }
    xi_row[k] = s0; xti_row[k] = s1;
}

// ------------------------------------------------------------------------------------------
// Walk kernel: grid = column tiles; one launch per batch.  Eq. (1) couples workers but never
// coordinates, so a workgroup that owns a tile of columns can apply EVERY operation of the batch
// to that tile, in the batch's (level-sorted, hence per-worker serial) order, without
// synchronising with any other workgroup: all accesses of a lane hit the lane's own columns and
// a wave's accesses to one address are performed in program order.  Compared with one launch
// per level this removes the drain/fill bubble between levels, which matters because most levels
// of a greedily packed batch hold far fewer than n/2 operations.  Every operation still reads and
// writes its rows from and to memory (the tiles of all resident workgroups together exceed the
// caches by far), so the traffic is the same 32 d / 16-24 d bytes per event.
// Operation records are uniform per workgroup and are fetched with scalar loads.
// Measured fastest on MI355X with TPB = 256, U = 1 and ordinary (temporal) accesses.  Applying two operations on
// disjoint workers in one pass, with the loads of both in flight together, was measured as well and gains nothing on
// the event streams (ring: +-0 %, exponential and complete graph: -1 to -3 %), although a plain in-place pass over
// four rows at a time streams faster than one over two.
// ------------------------------------------------------------------------------------------
template <int U, bool NT, int TPB>
__global__ __launch_bounds__(TPB) void walk_kernel(float *__restrict__ x, float *__restrict__ xt,
                                                   int64_t ld, int64_t d, const DevOp *__restrict__ ops,
                                                   int32_t n_ops, float alpha, float alpha_t) {
    extern __shared__ unsigned char occupancy_ballast[];     // never touched: its size limits the workgroups per CU
    const int64_t tile = blockIdx.x;
    for (int32_t k = 0; k < n_ops; ++k) {
        const DevOp op = ops[k];
        apply_op_tile<U, NT, TPB>(x, xt, ld, d, op, tile, alpha, alpha_t);
    }
}


// The coefficients of one operation, as the update functions read them.
struct OpCoef { float b_i, b_j, bp_i, bp_j, gamma, gscale; };

// ------------------------------------------------------------------------------------------
// Chain kernel: the walk, on a programme the host has ordered and annotated (plan_chain).  Any linear
// extension of the per-worker orders gives the same result bit for bit (operations on disjoint rows
// commute exactly), so the host picks one in which an operation finds its workers' columns close by
// as often as possible, and tells the kernel where each row comes from and goes to:
//   - the carry registers: a worker shared by two consecutive operations is neither stored by the
//     first nor loaded by the second (70-80 % of the operations on the paper's graphs).  The carried
//     worker is always presented as row_i; swapping the two ends of a gossip operation negates m,
//     which changes no bit of the result;
//   - an LDS slot: a worker with a pending operation is parked (2 x 16 bytes per lane and slot) instead
//     of stored, and read back from there; a spill pseudo-operation writes a parked worker to memory
//     when its slot is needed for a worker that comes back sooner (a worker's last operation of the
//     launch always leaves it in memory);
//   - device memory otherwise.
// A lane only ever touches its own LDS cells, so there is no barrier.  A gossip operation that gets
// one worker from the registers and hands one on moves 16 bytes per column instead of 32.
// Dynamic LDS: slots * U * TPB * 32 bytes.  The d % 4 trailing columns always go through memory.
// ------------------------------------------------------------------------------------------
// The two rows (x, xt) of a worker at location loc, memory or an LDS slot, for the lanes' pieces of the tile.
template <int U, int TPB>
__device__ __forceinline__ void chain_fetch(uint32_t loc, int32_t row, v4f (&v)[U], v4f (&vt)[U], const v4f *xs,
                                            const v4f *xts, int64_t ld4, const v4f *parked, const uint32_t (&lp)[U],
                                            const bool (&act)[U]) {
    if (loc == kLocMemory) {
        const v4f *p = xs + (int64_t)row * ld4, *pt = xts + (int64_t)row * ld4;
#pragma unroll
        for (int u = 0; u < U; ++u)
            if (act[u]) { v[u] = p[lp[u]]; vt[u] = pt[lp[u]]; }
    } else {
        const v4f *s = parked + (size_t)(loc - kLocSlot0) * (2 * U * TPB);
#pragma unroll
        for (int u = 0; u < U; ++u) { v[u] = s[lp[u]]; vt[u] = s[U * TPB + lp[u]]; }
    }
}

template <int U, int TPB>
__device__ __forceinline__ void chain_put(uint32_t loc, int32_t row, const v4f (&v)[U], const v4f (&vt)[U], v4f *xs,
                                          v4f *xts, int64_t ld4, v4f *parked, const uint32_t (&lp)[U],
                                          const bool (&act)[U]) {
    if (loc == kLocMemory) {
        v4f *p = xs + (int64_t)row * ld4, *pt = xts + (int64_t)row * ld4;
#pragma unroll
        for (int u = 0; u < U; ++u)
            if (act[u]) { p[lp[u]] = v[u]; pt[lp[u]] = vt[u]; }
    } else {
        v4f *s = parked + (size_t)(loc - kLocSlot0) * (2 * U * TPB);
#pragma unroll
        for (int u = 0; u < U; ++u) { s[lp[u]] = v[u]; s[U * TPB + lp[u]] = vt[u]; }
    }
}

template <int U, int TPB>
__global__ __launch_bounds__(TPB) void chain_kernel(float *__restrict__ x, float *__restrict__ xt, int64_t ld,
                                                    int64_t d, const DevOp *__restrict__ ops, int32_t n_ops,
                                                    float alpha, float alpha_t) {
    extern __shared__ v4f parked[];                      // [slot][x | xt][U][TPB]
    // a row's pieces of this tile are at (row base + tile0, a workgroup-uniform address) + lane-dependent
    // 32-bit offsets: scalar base plus vector offset, no 64-bit address arithmetic per lane
    const int64_t tile0 = (int64_t)blockIdx.x * (U * TPB);          // first float4 piece of the tile
    const int64_t left = (d >> 2) - tile0;                          // whole pieces from there to the row's end
    uint32_t lp[U];
    bool act[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
        lp[u] = (uint32_t)(u * TPB) + threadIdx.x;
        act[u] = (int64_t)lp[u] < left;
    }
    v4f *const xs = (v4f *)x + tile0, *const xts = (v4f *)xt + tile0;
    const int64_t ld4 = ld >> 2;
    const v4f zero = {0.f, 0.f, 0.f, 0.f};
    v4f a[U], at[U];                                     // row_i's columns; the carry registers between operations
#pragma unroll
    for (int u = 0; u < U; ++u) { a[u] = zero; at[u] = zero; }

    for (int32_t k = 0; k < n_ops; ++k) {
        // field by field: the record stays in scalar registers
        const DevOp *rec = ops + k;
        const int32_t word = rec->kind, row_i = rec->row_i, row_j = rec->row_j;
        const int32_t kind = op_kind(word);
        const uint32_t loc = rec->loc;
        const uint32_t src_i = loc & 255u, src_j = (loc >> 8) & 255u, dst_i = (loc >> 16) & 255u, dst_j = loc >> 24;
        if (kind == kOpSpill) {                          // a parked worker goes back to memory
            v4f b[U], bt[U];
            chain_fetch<U, TPB>(src_i, row_i, b, bt, xs, xts, ld4, parked, lp, act);
            chain_put<U, TPB>(kLocMemory, row_i, b, bt, xs, xts, ld4, parked, lp, act);
            continue;
        }
        const bool pre = (op_flags(word) & kFlagListing) != 0;
        const OpCoef oc = {rec->b_i, rec->b_j, rec->bp_i, rec->bp_j, rec->gamma, rec->gscale};
        if (src_i != kLocCarry) chain_fetch<U, TPB>(src_i, row_i, a, at, xs, xts, ld4, parked, lp, act);
        if (kind == kOpGossip) {
            v4f b[U], bt[U];
#pragma unroll
            for (int u = 0; u < U; ++u) { b[u] = zero; bt[u] = zero; }
            chain_fetch<U, TPB>(src_j, row_j, b, bt, xs, xts, ld4, parked, lp, act);
#pragma unroll
            for (int u = 0; u < U; ++u) gossip_update(a[u], at[u], b[u], bt[u], oc, alpha, alpha_t, pre);
            if (dst_j == kLocCarry) {
                chain_put<U, TPB>(dst_i, row_i, a, at, xs, xts, ld4, parked, lp, act);   // never the registers as well
#pragma unroll
                for (int u = 0; u < U; ++u) { a[u] = b[u]; at[u] = bt[u]; }
            } else {
                chain_put<U, TPB>(dst_j, row_j, b, bt, xs, xts, ld4, parked, lp, act);
                if (dst_i != kLocCarry) chain_put<U, TPB>(dst_i, row_i, a, at, xs, xts, ld4, parked, lp, act);
            }
        } else {
            if (kind == kOpGradient) {
                const float *xi = rec->xi, *cc = rec->c, *hh = rec->h;
                const bool has_xi = xi != nullptr;
                const bool has_c = cc != nullptr && oc.gscale != 0.f;
                const bool has_h = hh != nullptr && oc.gscale != 0.f;
                const v4f *pxi = (const v4f *)xi + tile0, *pc = (const v4f *)cc + tile0, *ph = (const v4f *)hh + tile0;
                const v4f one = {1.f, 1.f, 1.f, 1.f};
                v4f g[U], c[U], h[U];
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    g[u] = (has_xi && act[u]) ? load4<true>(pxi + lp[u]) : zero;
                    c[u] = (has_c && act[u]) ? load4<true>(pc + lp[u]) : zero;
                    h[u] = (has_h && act[u]) ? load4<true>(ph + lp[u]) : one;
                }
#pragma unroll
                for (int u = 0; u < U; ++u) gradient_update(a[u], at[u], g[u], c[u], h[u], oc, pre);
            } else {
#pragma unroll
                for (int u = 0; u < U; ++u) mix(a[u], at[u], oc.b_i);
            }
            if (dst_i != kLocCarry) chain_put<U, TPB>(dst_i, row_i, a, at, xs, xts, ld4, parked, lp, act);
        }
        if (blockIdx.x == 0) apply_op_tail(x, xt, ld, d, *rec, alpha, alpha_t);
    }
}

typedef const __attribute__((address_space(1))) float *global_f32;

__device__ __forceinline__ uint32_t lane_u32(uint32_t v, int l) { return (uint32_t)__builtin_amdgcn_readlane((int)v, l); }
__device__ __forceinline__ float lane_f32(uint32_t v, int l) { return __int_as_float(__builtin_amdgcn_readlane((int)v, l)); }

// C consecutive floats of a row starting at column col (col is a multiple of C, rows are 16-byte aligned);
// columns at or beyond d read as 0 and are never written.
template <int C>
struct Cols { float v[C]; };

template <int C>
__device__ __forceinline__ Cols<C> load_cols(const float *p, int64_t col, int64_t d) {
    typedef float vec __attribute__((ext_vector_type(C)));
    Cols<C> r;
    if (col + C <= d) {
        if constexpr (C == 1) r.v[0] = p[col];
        else { const vec t = *(const vec *)(p + col);
#pragma unroll
               for (int c = 0; c < C; ++c) r.v[c] = t[c]; }
    } else {
#pragma unroll
        for (int c = 0; c < C; ++c) r.v[c] = col + c < d ? p[col + c] : 0.f;
    }
    return r;
}

template <int C>
__device__ __forceinline__ void store_cols(float *p, int64_t col, int64_t d, const Cols<C> &r) {
    typedef float vec __attribute__((ext_vector_type(C)));
    if (col + C <= d) {
        if constexpr (C == 1) p[col] = r.v[0];
        else { vec t;
#pragma unroll
               for (int c = 0; c < C; ++c) t[c] = r.v[c];
               *(vec *)(p + col) = t; }
    } else {
#pragma unroll
        for (int c = 0; c < C; ++c) if (col + c < d) p[col + c] = r.v[c];
    }
}

// ------------------------------------------------------------------------------------------
// Resident kernel: grid = tiles of 64 * C columns, W waves per workgroup, one launch per batch (or per piece of
// a batch).  The same ownership argument as for the walk kernel, taken one step further: the workgroup first
// copies its columns of every row the launch touches into LDS, then applies all operations of the launch to the
// LDS copy, and finally writes the rows back.  State traffic per launch drops from 32 d bytes per gossip event to
// 16 d bytes per touched row; gradient inputs are still read once per event.
//
// LDS capacity allows only a few such tiles per CU, so the W waves of a workgroup share one tile: lane l of every
// wave stands for columns l*C .. l*C+C-1 of the tile, the operations of a level (which touch disjoint rows) are
// dealt to the waves, and a workgroup barrier separates levels.  The kernel is bound by instruction issue, not
// by memory or LDS bandwidth, so everything a wave can be spared is done on the host, which writes one linear
// programme per wave:
//   - the programme is typed by position: a control slot says how many gossip operations and then how many
//     gradient operations follow, so the operation loops test no kind, and operations carry ready-made LDS
//     byte offsets of their rows;
//   - a programme is at most 256 or 512 slots of 16 bytes (resident_slots), and a wave holds all of it in
//     registers from the start (four or eight slots per lane): the operation loops read their operands with
//     v_readlane and never touch memory for them.  The host cuts a batch into launches whose programmes fit, and
//     never lets a level straddle a set of 64 slots (it closes a set early with a jump slot), so the loops over
//     one set are plain;
//   - gradient inputs do not pass through LDS and need no barrier of their own: every gradient operation names
//     the wave's NEXT gradient event (its xi pointer in the slot, c and h through the gin table), and the wave
//     requests those inputs into registers as soon as it has used the current ones; the host deals the
//     gradient events of a level to the waves whose last one lies furthest back, so a request has several
//     levels' time to arrive.  The very first ones are named by the programme's first control slot.
// Whether jumps are taken from the stored values (PRE: Algorithm 1 as listed), whether any operation of the
// launch carries a trailing mix (TRAIL) and whether any gradient event has a centre c (HC) or a curvature h (HH)
// are compile-time cases, so the common path carries no test and no load for them.
// Valid only while every gradient input of the batch is final when the batch is submitted (true for the affine
// gradient model; a real network's gradient at x_i is not).  Its throughput is reported apart from the roofline
// of the one-pass-per-event kernels: it is not bound by memory.
// LDS: n_rows * 64 * 8 C bytes (C = 1: (x, xt) pairs; C = 2, 4: planes of 16-byte cells holding two columns).
// ------------------------------------------------------------------------------------------
// Slot layout, control codes and sizes: a2cid_internal.h (shared with the planner).

typedef float v2f __attribute__((ext_vector_type(2)));

// The lane's C columns of a row (x and xt) to and from its cell(s) at LDS byte offset off (which already includes
// the lane's own offset): C = 1: one (x, xt) pair; C = 2, 4: cells (x, xt, x', xt') of two columns, one per plane.
template <int C>
__device__ __forceinline__ void res_put(unsigned char *lds, uint32_t off, const Cols<C> &a, const Cols<C> &at) {
    if constexpr (C == 1) {
        const v2f t = {a.v[0], at.v[0]};
        *(v2f *)(lds + off) = t;
    } else {
#pragma unroll
        for (int h = 0; h < C / 2; ++h) {
            const v4f t = {a.v[2 * h], at.v[2 * h], a.v[2 * h + 1], at.v[2 * h + 1]};
            *(v4f *)(lds + off + h * 1024) = t;
        }
    }
}

template <int C>
__device__ __forceinline__ void res_get(const unsigned char *lds, uint32_t off, Cols<C> &a, Cols<C> &at) {
    if constexpr (C == 1) {
        const v2f t = *(const v2f *)(lds + off);
        a.v[0] = t.x; at.v[0] = t.y;
    } else {
#pragma unroll
        for (int h = 0; h < C / 2; ++h) {
            const v4f t = *(const v4f *)(lds + off + h * 1024);
            a.v[2 * h] = t.x; at.v[2 * h] = t.y; a.v[2 * h + 1] = t.z; at.v[2 * h + 1] = t.w;
        }
    }
}

// Columns col0 + lane_c .. + C - 1 of one gradient input.  whole: every lane of the tile has C columns below d.
// The input is addressed as global memory (a generic pointer would make these loads count as possible LDS
// accesses, and every LDS access of the operation loops would then wait for them).
template <int C>
__device__ __forceinline__ void res_input(float (&out)[C], uintptr_t p, int64_t col0, uint32_t lane_c, int64_t d,
                                         bool whole, float absent) {
    typedef float vec __attribute__((ext_vector_type(C)));
    typedef const __attribute__((address_space(1))) vec *global_vec;
    if (p & 1) {                                          // no row: the constant 0 (tag 1) or 1 (tag 3) for every column
        const float z = (p & 2) ? 1.f : 0.f;
#pragma unroll
        for (int c = 0; c < C; ++c) out[c] = z;
        return;
    }
    const global_f32 base = (global_f32)p + col0;         // uniform; the lane adds a 32-bit offset
    if (whole) {
        if constexpr (C == 1) out[0] = __builtin_nontemporal_load(base + lane_c);
        else {
            const vec t = __builtin_nontemporal_load((global_vec)(base + lane_c));
#pragma unroll
            for (int c = 0; c < C; ++c) out[c] = t[c];
        }
    } else {
#pragma unroll
        for (int c = 0; c < C; ++c) out[c] = col0 + lane_c + c < d ? base[lane_c + c] : absent;
    }
}

template <int C, bool HC, bool HH>
__device__ __forceinline__ void res_request(float (&gx)[C], float (&gc)[C], float (&gh)[C], uint32_t xi_lo,
                                           uint32_t xi_hi, const GradIn *__restrict__ gin, uint32_t g, int64_t col0,
                                           uint32_t lane_c, int64_t d, bool whole) {
    res_input<C>(gx, (uintptr_t)xi_lo | (uintptr_t)xi_hi << 32, col0, lane_c, d, whole, 0.f);
    if constexpr (HC) res_input<C>(gc, gin[g].c, col0, lane_c, d, whole, 0.f);
    if constexpr (HH) res_input<C>(gh, gin[g].h, col0, lane_c, d, whole, 1.f);
}

template <int W, int C, bool PRE, bool TRAIL, bool HC, bool HH>
__global__ __launch_bounds__(64 * W) void resident_kernel(float *__restrict__ x, float *__restrict__ xt, int64_t ld,
                                                           int64_t d, const ResSlot *__restrict__ recs,
                                                           const GradIn *__restrict__ gin,
                                                           const int32_t *__restrict__ rows, int32_t n_rows,
                                                           float alpha, float alpha_t) {
    extern __shared__ unsigned char lds[];
    constexpr uint32_t kCell = C == 1 ? 8 : 16;
    constexpr uint32_t kRow = resident_row_bytes(C);
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int64_t col0 = (int64_t)blockIdx.x * (64 * C);            // first column of the tile (uniform)
    const uint32_t lane_c = (uint32_t)lane * C;
    const int64_t col = col0 + lane_c;
    const bool valid = col < d;
    const bool whole = col0 + 64 * C <= d;
    const uint32_t lane_off = (uint32_t)lane * kCell;

    // this wave's whole programme: slot 64 k + lane in set k
    constexpr int kSets = resident_sets(W);
    const uint4 *prog = (const uint4 *)recs + (size_t)wave * (64 * kSets) + lane;
    uint4 set[kSets];
#pragma unroll
    for (int k = 0; k < kSets; ++k) set[k] = prog[64 * k];

    // the wave's first gradient inputs
    float gx[C], gc[C], gh[C];
#pragma unroll
    for (int c = 0; c < C; ++c) { gx[c] = 0.f; gc[c] = 0.f; gh[c] = 1.f; }
    {
        const uint32_t g0 = lane_u32(set[0].y, 0);
        if (g0 != kResNone)
            res_request<C, HC, HH>(gx, gc, gh, lane_u32(set[0].z, 0), lane_u32(set[0].w, 0), gin, g0, col0, lane_c, d, whole);
    }

    // rows wave, wave + W, ... of the slot list into LDS, four rows' loads in flight per wave
    for (int32_t s0 = wave; s0 < n_rows; s0 += 4 * W) {
        Cols<C> a[4], at[4];
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const int32_t s = s0 + q * W;
#pragma unroll
            for (int c = 0; c < C; ++c) { a[q].v[c] = 0.f; at[q].v[c] = 0.f; }
            if (s < n_rows && valid) {
                const int64_t off = (int64_t)rows[s] * ld;
                a[q] = load_cols<C>(x + off, col, d);
                at[q] = load_cols<C>(xt + off, col, d);
            }
        }
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const int32_t s = s0 + q * W;
            if (s < n_rows) res_put<C>(lds, (uint32_t)s * kRow + lane_off, a[q], at[q]);
        }
    }
    // Every load issued so far (programme, rows, first gradient inputs) is waited for here, once: the compiler then
    // knows that no register has a load pending when the operation loops begin, and puts no wait for vector
    // memory into them except where requested gradient inputs are used (s_waitcnt vmcnt(0) expcnt(7) lgkmcnt(15)).
    __builtin_amdgcn_s_waitcnt(0x0F70);
    // no barrier here: every programme starts with a level slot, which brings one

    // The slots of one set, from its first to a jump slot (returns false) or to the end of the programme (true).
    auto run_set = [&](const uint4 &r) __attribute__((always_inline)) -> bool {
        int32_t pos = 0;                                 // lane that holds the next slot
        for (;;) {
            const uint32_t w0 = lane_u32(r.x, pos);
            if (w0 >= kResJump) return w0 != kResJump;
            const int32_t n_gossip = (int32_t)(w0 & 255u), n_grad = (int32_t)(w0 >> 8);
            ++pos;
            __syncthreads();                             // the previous level is complete in LDS
            int32_t t = 0;
            if constexpr (C == 1) {
                // two operations of the level at a time (they touch disjoint rows): one LDS round trip for both
                constexpr int kStep = TRAIL ? 2 : 1;
                for (; t + 2 <= n_gossip; t += 2, pos += 2 * kStep) {
                    const int32_t p2 = pos + kStep;
                    const uint32_t oi = lane_u32(r.x, pos) + lane_off, oj = lane_u32(r.y, pos) + lane_off;
                    const uint32_t oi2 = lane_u32(r.x, p2) + lane_off, oj2 = lane_u32(r.y, p2) + lane_off;
                    v2f a = *(const v2f *)(lds + oi), b = *(const v2f *)(lds + oj);
                    v2f a2 = *(const v2f *)(lds + oi2), b2 = *(const v2f *)(lds + oj2);
                    OpCoef oc, oc2;
                    oc.b_i = lane_f32(r.z, pos); oc.b_j = lane_f32(r.w, pos);
                    oc.bp_i = TRAIL ? lane_f32(r.x, pos + 1) : 0.f;
                    oc.bp_j = TRAIL ? lane_f32(r.y, pos + 1) : 0.f;
                    oc2.b_i = lane_f32(r.z, p2); oc2.b_j = lane_f32(r.w, p2);
                    oc2.bp_i = TRAIL ? lane_f32(r.x, p2 + 1) : 0.f;
                    oc2.bp_j = TRAIL ? lane_f32(r.y, p2 + 1) : 0.f;
                    float xi_ = a.x, xti = a.y, xj = b.x, xtj = b.y;
                    float xi2 = a2.x, xti2 = a2.y, xj2 = b2.x, xtj2 = b2.y;
                    gossip_jump<TRAIL>(xi_, xti, xj, xtj, oc, alpha, alpha_t, PRE);
                    gossip_jump<TRAIL>(xi2, xti2, xj2, xtj2, oc2, alpha, alpha_t, PRE);
                    a.x = xi_; a.y = xti; b.x = xj; b.y = xtj;
                    a2.x = xi2; a2.y = xti2; b2.x = xj2; b2.y = xtj2;
                    *(v2f *)(lds + oi) = a;
                    *(v2f *)(lds + oj) = b;
                    *(v2f *)(lds + oi2) = a2;
                    *(v2f *)(lds + oj2) = b2;
                }
            }
            for (; t < n_gossip; ++t, pos += TRAIL ? 2 : 1) {
                const uint32_t oi = lane_u32(r.x, pos) + lane_off, oj = lane_u32(r.y, pos) + lane_off;
                OpCoef oc;
                oc.b_i = lane_f32(r.z, pos); oc.b_j = lane_f32(r.w, pos);
                oc.bp_i = TRAIL ? lane_f32(r.x, pos + 1) : 0.f;
                oc.bp_j = TRAIL ? lane_f32(r.y, pos + 1) : 0.f;
                if constexpr (C == 1) {
                    v2f a = *(const v2f *)(lds + oi), b = *(const v2f *)(lds + oj);
                    float xi_ = a.x, xti = a.y, xj = b.x, xtj = b.y;
                    gossip_jump<TRAIL>(xi_, xti, xj, xtj, oc, alpha, alpha_t, PRE);
                    a.x = xi_; a.y = xti; b.x = xj; b.y = xtj;
                    *(v2f *)(lds + oi) = a;
                    *(v2f *)(lds + oj) = b;
                } else {
                    v4f a[C / 2], b[C / 2];              // all reads first: one LDS round trip per operation
#pragma unroll
                    for (int h = 0; h < C / 2; ++h) {
                        a[h] = *(const v4f *)(lds + oi + h * 1024);
                        b[h] = *(const v4f *)(lds + oj + h * 1024);
                    }
#pragma unroll
                    for (int h = 0; h < C / 2; ++h) {
                        float i0 = a[h].x, it0 = a[h].y, i1 = a[h].z, it1 = a[h].w;
                        float j0 = b[h].x, jt0 = b[h].y, j1 = b[h].z, jt1 = b[h].w;
                        gossip_jump<TRAIL>(i0, it0, j0, jt0, oc, alpha, alpha_t, PRE);
                        gossip_jump<TRAIL>(i1, it1, j1, jt1, oc, alpha, alpha_t, PRE);
                        const v4f na = {i0, it0, i1, it1}, nb = {j0, jt0, j1, jt1};
                        a[h] = na; b[h] = nb;
                    }
#pragma unroll
                    for (int h = 0; h < C / 2; ++h) {
                        *(v4f *)(lds + oi + h * 1024) = a[h];
                        *(v4f *)(lds + oj + h * 1024) = b[h];
                    }
                }
            }
            for (int32_t t = 0; t < n_grad; ++t, pos += 2) {
                const uint32_t oi = lane_u32(r.x, pos) + lane_off;
                OpCoef oc;
                oc.b_i = lane_f32(r.y, pos); oc.gamma = lane_f32(r.z, pos); oc.gscale = lane_f32(r.w, pos);
                oc.bp_i = TRAIL ? lane_f32(r.y, pos + 1) : 0.f;
                if constexpr (C == 1) {
                    v2f a = *(const v2f *)(lds + oi);
                    float xi_ = a.x, xti = a.y;
                    gradient_jump<TRAIL>(xi_, xti, gx[0], gc[0], gh[0], oc, PRE);
                    a.x = xi_; a.y = xti;
                    *(v2f *)(lds + oi) = a;
                } else {
                    v4f a[C / 2];
#pragma unroll
                    for (int h = 0; h < C / 2; ++h) a[h] = *(const v4f *)(lds + oi + h * 1024);
#pragma unroll
                    for (int h = 0; h < C / 2; ++h) {
                        float i0 = a[h].x, it0 = a[h].y, i1 = a[h].z, it1 = a[h].w;
                        gradient_jump<TRAIL>(i0, it0, gx[2 * h], gc[2 * h], gh[2 * h], oc, PRE);
                        gradient_jump<TRAIL>(i1, it1, gx[2 * h + 1], gc[2 * h + 1], gh[2 * h + 1], oc, PRE);
                        const v4f na = {i0, it0, i1, it1};
                        a[h] = na;
                    }
#pragma unroll
                    for (int h = 0; h < C / 2; ++h) *(v4f *)(lds + oi + h * 1024) = a[h];
                }
                const uint32_t next = lane_u32(r.x, pos + 1);
                if (next != kResNone)
                    res_request<C, HC, HH>(gx, gc, gh, lane_u32(r.z, pos + 1), lane_u32(r.w, pos + 1), gin, next, col0,
                                           lane_c, d, whole);
            }
        }
    };
#pragma unroll
    for (int k = 0; k < kSets; ++k)
        if (run_set(set[k])) break;                      // the last set always ends the programme
    __syncthreads();

    if (valid) {
        for (int32_t s = wave; s < n_rows; s += W) {
            Cols<C> a, at;
            res_get<C>(lds, (uint32_t)s * kRow + lane_off, a, at);
            const int64_t off = (int64_t)rows[s] * ld;
            store_cols<C>(x + off, col, d, a);
            store_cols<C>(xt + off, col, d, at);
        }
    }
}

// ------------------------------------------------------------------------------------------
// Register-file kernel: grid = tiles of 64 columns, one wave per workgroup, one launch per batch (or piece of one).
// The ownership argument taken to its end: with at most 64 workers a lane can hold its column of EVERY worker's x
// and xt in vector registers (worker r: v[r] and v[64 + r]), so a wave loads its 64 columns of the touched rows once,
// applies the whole programme to registers and stores the rows back: no LDS, no barrier, nothing shared between waves
// but the (read-only) programme.  Which register an operation touches is only known at run time, so the operations
// address the register file relatively: S_SET_GPR_IDX_ON adds a scalar index (the low 8 bits of its operand) to
// chosen operands of the vector instructions that follow, here to the operands written as v0 (x), v64 (xt) and
// v128 / v144 / v160 (gradient inputs).  Only s_set_gpr_idx_on / s_set_gpr_idx_off bracket the indexed instructions,
// the forms the compiler itself emits for dynamically indexed vectors.
//
// The operation loop is one asm statement with a fixed register map, because the register allocator cannot be made
// to keep four 32-register blocks in place across compiler-visible control flow (it begins with the row loads; the
// row stores after it are a second statement on the same pinned registers):
//   v[0:63] x, v[64:127] xt of the 64 workers (the statement's in/out operands, pinned by their constraints)
//   v[128:135], v[136:143]   the two sets of gradient inputs xi (kRegChunk events each)
//   with centres: v[144:151], v[152:159] the sets of centres c; with curvatures also v[160:167], v[168:175] for h
//   v[TB .. TB+6]            temporaries (TB = 144, with centres 160, with curvatures 176)
//   s[36:67], s[68:99] two blocks of 8 slots (one applied, one being fetched), s26 byte position of the next fetch,
//   s27, s31 scratch, s28 index of the next gradient event's inputs (set offset included), s29 offset of the set in
//   use (0 or 8), s30 (with centres) set while the block of c and h pointers after a request is to be passed over
// Programme (layout: a2cid_internal.h): every slot is applied in order; a gossip slot (the common case) falls
// through its kind test, the other kinds are handled out of line.  The loop ends at the end slot, and in any case
// when the position reaches the programme's length.
// Gradient inputs: chunk k of kRegChunk events uses set k % 2.  The pointers travel in the programme itself, in
// request blocks (8 xi pointers in slots 1-4; with centres the block after it holds 8 c and 8 h pointers), so they arrive
// with the block prefetch.  The programme begins with the request blocks of chunks 0 and 1.  The request block of
// chunk k + 1 precedes the first event of chunk k >= 1; its first slot is a switch slot: the wave waits for chunk k's
// set (requested a whole chunk ago; nothing else is in flight), requests chunk k + 1 into the set chunk k - 1 used,
// turns to chunk k's set and goes on with the next block.  A pointer with bit 0 set is the address of one float
// that stands for every column (an absent input, or an event past the last).
// The arithmetic is the shared sequence of individually rounded operations (mix, gossip_jump, gradient_jump: the
// same subtractions and fused multiply-adds in the same order), so results agree bit for bit with the other kernels.
// Valid only while every gradient input of the batch is final when the batch is submitted, like the resident kernel.
// ------------------------------------------------------------------------------------------
typedef float v32f __attribute__((ext_vector_type(32)));

// A uniform address as the compiler must take it: a value in scalar registers.
__device__ __forceinline__ uintptr_t reg_uniform(const float *p) {
    const uintptr_t v = (uintptr_t)p;
    const uint32_t lo = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)v);
    const uint32_t hi = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)(v >> 32));
    return (uintptr_t)lo | (uintptr_t)hi << 32;
}

#define A2R_T(TB, k) "v[" TB "+" #k "]"
#define A2R_ON(idx, mode) "s_set_gpr_idx_on " idx ", gpr_idx(" mode ")\n\t"
#define A2R_OFF "s_set_gpr_idx_off\n\t"
// temporaries: 0 di, 1 dj (gradient: g), 2 xi, 3 ti, 4 xj (gradient: u / stored x), 5 tj (gradient: slope), 6 m (request:
// the lane's offset)
// Index mode stays on from one operation to the next (every vector instruction of an operation comes after the
// operation's own s_set_gpr_idx_on); it is switched off before the only other vector instructions, those of a
// request, and at the end.

// mix of workers X (i) and Y (j) to the event time, difference m, the four jumps; Z = b_i, W = b_j
#define A2R_GOSSIP_MIX(TB, X, Y, Z, W)                                                                              \
    A2R_ON(X, "SRC0,SRC1") "v_sub_f32 " A2R_T(TB, 0) ", v64, v0\n\t"                                                \
    A2R_ON(Y, "SRC0,SRC1") "v_sub_f32 " A2R_T(TB, 1) ", v64, v0\n\t"                                                \
    A2R_ON(X, "SRC2") "v_fma_f32 " A2R_T(TB, 2) ", " Z ", " A2R_T(TB, 0) ", v0\n\t"                                 \
                      "v_fma_f32 " A2R_T(TB, 3) ", -" Z ", " A2R_T(TB, 0) ", v64\n\t"                               \
    A2R_ON(Y, "SRC2") "v_fma_f32 " A2R_T(TB, 4) ", " W ", " A2R_T(TB, 1) ", v0\n\t"                                 \
                      "v_fma_f32 " A2R_T(TB, 5) ", -" W ", " A2R_T(TB, 1) ", v64\n\t"
#define A2R_GOSSIP_JUMP(TB, X, Y)                                                                                   \
    A2R_ON(X, "DST") "v_fma_f32 v0, %[nal], " A2R_T(TB, 6) ", " A2R_T(TB, 2) "\n\t"                                 \
                     "v_fma_f32 v64, %[nalt], " A2R_T(TB, 6) ", " A2R_T(TB, 3) "\n\t"                               \
    A2R_ON(Y, "DST") "v_fma_f32 v0, %[al], " A2R_T(TB, 6) ", " A2R_T(TB, 4) "\n\t"                                  \
                     "v_fma_f32 v64, %[alt], " A2R_T(TB, 6) ", " A2R_T(TB, 5) "\n\t"
// m after the mixing (Eq. (1)): a two-operand instruction, untouched by the SRC2 mode still in force
#define A2R_GOSSIP_0(TB, X, Y, Z, W)                                                                                \
    A2R_GOSSIP_MIX(TB, X, Y, Z, W)                                                                                  \
    "v_sub_f32 " A2R_T(TB, 6) ", " A2R_T(TB, 2) ", " A2R_T(TB, 4) "\n\t"                                            \
    A2R_GOSSIP_JUMP(TB, X, Y)
// m from the stored values (Algorithm 1 as listed)
#define A2R_GOSSIP_1(TB, X, Y, Z, W)                                                                                \
    A2R_ON(Y, "SRC0") "v_mov_b32 " A2R_T(TB, 6) ", v0\n\t"                                                          \
    A2R_ON(X, "SRC0") "v_sub_f32 " A2R_T(TB, 6) ", v0, " A2R_T(TB, 6) "\n\t"                                        \
    A2R_GOSSIP_MIX(TB, X, Y, Z, W)                                                                                  \
    A2R_GOSSIP_JUMP(TB, X, Y)

// gradient event of worker s31 (index), Y = b_i, Z = gamma, W = gscale; inputs at index s28
#define A2R_STORED_2(TB)
#define A2R_STORED_4(TB) A2R_ON("s31", "SRC0") "v_mov_b32 " A2R_T(TB, 4) ", v0\n\t"
#define A2R_GRAD_HEAD(TB, Y, AT)                                                                                    \
    A2R_ON("s31", "SRC0,SRC1") "v_sub_f32 " A2R_T(TB, 0) ", v64, v0\n\t"                                            \
    A2R_STORED_##AT(TB)                                                                                             \
    A2R_ON("s31", "SRC2") "v_fma_f32 " A2R_T(TB, 2) ", " Y ", " A2R_T(TB, 0) ", v0\n\t"                             \
                          "v_fma_f32 " A2R_T(TB, 3) ", -" Y ", " A2R_T(TB, 0) ", v64\n\t"
#define A2R_GRAD_TAIL(TB, Z)                                                                                        \
    A2R_ON("s31", "DST") "v_fma_f32 v0, -" Z ", " A2R_T(TB, 1) ", " A2R_T(TB, 2) "\n\t"                             \
                         "v_fma_f32 v64, -" Z ", " A2R_T(TB, 1) ", " A2R_T(TB, 3) "\n\t"                            \
    "s_add_u32 s28, s28, 1\n\t"
// g = gscale x + xi (no centre, no curvature); AT = 2: at the mixed point, 4: at the stored point
#define A2R_GRAD_PLAIN(TB, Y, Z, W, AT)                                                                             \
    A2R_GRAD_HEAD(TB, Y, AT)                                                                                        \
    A2R_ON("s28", "SRC2") "v_fma_f32 " A2R_T(TB, 1) ", " W ", " A2R_T(TB, AT) ", v128\n\t"                          \
    A2R_GRAD_TAIL(TB, Z)
// g = (gscale h) (x - c) + xi
#define A2R_GRAD_FULL(TB, Y, Z, W, AT)                                                                              \
    A2R_GRAD_HEAD(TB, Y, AT)                                                                                        \
    A2R_ON("s28", "SRC1") "v_sub_f32 " A2R_T(TB, 4) ", " A2R_T(TB, AT) ", v144\n\t"                                 \
                          "v_mul_f32 " A2R_T(TB, 5) ", " W ", v160\n\t"                                             \
    A2R_ON("s28", "SRC2") "v_fma_f32 " A2R_T(TB, 1) ", " A2R_T(TB, 5) ", " A2R_T(TB, 4) ", v128\n\t"                \
    A2R_GRAD_TAIL(TB, Z)
// g = gscale (x - c) + xi (centres, no curvature)
#define A2R_GRAD_HC(TB, Y, Z, W, AT)                                                                                \
    A2R_GRAD_HEAD(TB, Y, AT)                                                                                        \
    A2R_ON("s28", "SRC1") "v_sub_f32 " A2R_T(TB, 4) ", " A2R_T(TB, AT) ", v144\n\t"                                 \
    A2R_ON("s28", "SRC2") "v_fma_f32 " A2R_T(TB, 1) ", " W ", " A2R_T(TB, 4) ", v128\n\t"                           \
    A2R_GRAD_TAIL(TB, Z)
#define A2R_MIX(TB, Y)                                                                                              \
    A2R_ON("s31", "SRC0,SRC1") "v_sub_f32 " A2R_T(TB, 0) ", v64, v0\n\t"                                            \
    A2R_ON("s31", "SRC2,DST") "v_fma_f32 v0, " Y ", " A2R_T(TB, 0) ", v0\n\t"                                       \
                              "v_fma_f32 v64, -" Y ", " A2R_T(TB, 0) ", v64\n\t"

// one slot in line: a gossip operation falls through
#define A2R_SLOT(TB, GOSSIP, id, X, Y, Z, W)                                                                        \
    "s_cmp_lt_u32 " X ", 0x100\n\t"                                                                                 \
    "s_cbranch_scc0 L_o" id "_%=\n\t"                                                                               \
    GOSSIP(TB, X, Y, Z, W)                                                                                          \
    "\nL_d" id "_%=:\n\t"
// the other kinds of the same slot (x >> 8 = 1 gradient, 2 mix, 3 control: told apart by bits 9 and 8), out of line,
// up to the control slots
#define A2R_OTHER_HEAD(TB, GRAD, AT, id, X, Y, Z, W)                                                                \
    "\nL_o" id "_%=:\n\t"                                                                                           \
    "s_and_b32 s31, " X ", 0xff\n\t"                                                                                \
    "s_bitcmp0_b32 " X ", 9\n\t"                                                                                    \
    "s_cbranch_scc0 L_p" id "_%=\n\t"                                                                               \
    GRAD(TB, Y, Z, W, AT)                                                                                           \
    "s_branch L_d" id "_%=\n"                                                                                       \
    "L_p" id "_%=:\n\t"                                                                                             \
    "s_bitcmp0_b32 " X ", 8\n\t"                                                                                    \
    "s_cbranch_scc0 L_c" id "_%=\n\t"                                                                               \
    A2R_MIX(TB, Y)                                                                                                  \
    "s_branch L_d" id "_%=\n"                                                                                       \
    "L_c" id "_%=:\n\t"
// a control slot: the end, or filler; in the first slot of a block (FIRST) also a switch
#define A2R_OTHER(TB, GRAD, AT, PH, id, X, Y, Z, W)                                                                 \
    A2R_OTHER_HEAD(TB, GRAD, AT, id, X, Y, Z, W)                                                                    \
    "s_cmp_eq_u32 " Y ", 2\n\t"                                                                                     \
    "s_cbranch_scc1 L_end_%=\n\t"                                                                                   \
    "s_branch L_d" id "_%=\n\t"
#define A2R_OTHER_FIRST(TB, GRAD, AT, PH, id, X, Y, Z, W)                                                           \
    A2R_OTHER_HEAD(TB, GRAD, AT, id, X, Y, Z, W)                                                                    \
    "s_cmp_eq_u32 " Y ", 1\n\t"                                                                                     \
    "s_cbranch_scc1 L_sw" PH "_%=\n\t"                                                                              \
    "s_cmp_eq_u32 " Y ", 2\n\t"                                                                                     \
    "s_cbranch_scc1 L_end_%=\n\t"                                                                                   \
    "s_branch L_d" id "_%=\n\t"
// the eight slots of block A (s[36:67]) and of block B (s[68:99]); M0 for the first slot, M for the others
#define A2R_SLOTS_A(M0, M, ...)                                                                                     \
    M0(__VA_ARGS__, "a0", "s36", "s37", "s38", "s39") M(__VA_ARGS__, "a1", "s40", "s41", "s42", "s43")              \
    M(__VA_ARGS__, "a2", "s44", "s45", "s46", "s47") M(__VA_ARGS__, "a3", "s48", "s49", "s50", "s51")               \
    M(__VA_ARGS__, "a4", "s52", "s53", "s54", "s55") M(__VA_ARGS__, "a5", "s56", "s57", "s58", "s59")               \
    M(__VA_ARGS__, "a6", "s60", "s61", "s62", "s63") M(__VA_ARGS__, "a7", "s64", "s65", "s66", "s67")
#define A2R_SLOTS_B(M0, M, ...)                                                                                     \
    M0(__VA_ARGS__, "b0", "s68", "s69", "s70", "s71") M(__VA_ARGS__, "b1", "s72", "s73", "s74", "s75")              \
    M(__VA_ARGS__, "b2", "s76", "s77", "s78", "s79") M(__VA_ARGS__, "b3", "s80", "s81", "s82", "s83")               \
    M(__VA_ARGS__, "b4", "s84", "s85", "s86", "s87") M(__VA_ARGS__, "b5", "s88", "s89", "s90", "s91")               \
    M(__VA_ARGS__, "b6", "s92", "s93", "s94", "s95") M(__VA_ARGS__, "b7", "s96", "s97", "s98", "s99")

// one input: its pointer in s[P+2k : P+2k+1] (bit 0: one float for every column), destination v[B+k]
#define A2R_REQ1(TB, B, P, k)                                                                                       \
    "s_bitcmp1_b32 s[" P "+2*" #k "], 0\n\t"                                                                        \
    "s_cselect_b64 vcc, -1, 0\n\t"                                                                                  \
    "v_cndmask_b32_e64 " A2R_T(TB, 6) ", %[voff], 0, vcc\n\t"                                                      \
    "s_and_b32 s[" P "+2*" #k "], s[" P "+2*" #k "], -4\n\t"                                                        \
    "global_load_dword v[" B "+" #k "], " A2R_T(TB, 6) ", s[" P "+2*" #k ":" P "+2*" #k "+1] nt\n\t"
// eight inputs of one kind: pointers in s[P : P+15], destinations v[B : B+7]
#define A2R_REQ8(TB, B, P)                                                                                          \
    A2R_REQ1(TB, B, P, 0) A2R_REQ1(TB, B, P, 1) A2R_REQ1(TB, B, P, 2) A2R_REQ1(TB, B, P, 3)                         \
    A2R_REQ1(TB, B, P, 4) A2R_REQ1(TB, B, P, 5) A2R_REQ1(TB, B, P, 6) A2R_REQ1(TB, B, P, 7)
// A request block: slot 0 a control slot, slots 1-4 the xi pointers of a chunk.  With centres and curvatures (FULL)
// the block after it holds the c pointers (slots 0-3) and the h pointers (slots 4-7).  XI: first SGPR of slot 1 of
// the request block, C / H: first SGPR of slots 0 / 4 of the other block; SET: "0" or "8".
#define A2R_REQ_PLAIN(TB, SET, XI, C, H) A2R_REQ8(TB, "128+" SET, XI)
#define A2R_REQ_HC(TB, SET, XI, C, H) A2R_REQ8(TB, "128+" SET, XI) A2R_REQ8(TB, "144+" SET, C)
#define A2R_REQ_FULL(TB, SET, XI, C, H)                                                                             \
    A2R_REQ8(TB, "128+" SET, XI) A2R_REQ8(TB, "144+" SET, C) A2R_REQ8(TB, "160+" SET, H)
// After a request with centres and curvatures the block of c and h pointers is passed over (s30 = 1: skip a block).
#define A2R_SKIP_SET_PLAIN
#define A2R_SKIP_SET_FULL "s_mov_b32 s30, 1\n\t"
#define A2R_SKIP_SET_HC A2R_SKIP_SET_FULL
#define A2R_SKIP_TEST_PLAIN(PH)
#define A2R_SKIP_TEST_FULL(PH)                                                                                      \
    "s_cmp_eq_u32 s30, 0\n\t"                                                                                       \
    "s_cbranch_scc1 L_go" PH "_%=\n\t"                                                                              \
    "s_mov_b32 s30, 0\n\t"                                                                                          \
    "s_branch L_end" PH "_%=\n"                                                                                     \
    "L_go" PH "_%=:\n\t"
#define A2R_SKIP_TEST_HC(PH) A2R_SKIP_TEST_FULL(PH)
// A switch slot (first slot of a block, phase PH): the wave waits for the set of inputs requested a chunk ago
// (nothing else is in flight; with centres and curvatures also for the block of their pointers, being fetched),
// requests the pointers of this block into the set just used up, turns to the other set and goes on with the
// next block.
#define A2R_SWITCH(TB, PH, REQ, VARIANT, XI, C, H)                                                                  \
    "\nL_sw" PH "_%=:\n\t"                                                                                          \
    A2R_OFF                                                                                                         \
    "s_waitcnt vmcnt(0) lgkmcnt(0)\n\t"                                                                             \
    "s_cmp_eq_u32 s29, 0\n\t"                                                                                       \
    "s_cbranch_scc0 L_sw" PH "b_%=\n\t"                                                                             \
    REQ(TB, "0", XI, C, H)                                                                                          \
    "s_mov_b32 s29, 8\n\t"                                                                                          \
    "s_mov_b32 s28, 8\n\t"                                                                                          \
    A2R_SKIP_SET_##VARIANT                                                                                          \
    "s_branch L_end" PH "_%=\n"                                                                                     \
    "L_sw" PH "b_%=:\n\t"                                                                                           \
    REQ(TB, "8", XI, C, H)                                                                                          \
    "s_mov_b32 s29, 0\n\t"                                                                                          \
    "s_mov_b32 s28, 0\n\t"                                                                                          \
    A2R_SKIP_SET_##VARIANT                                                                                          \
    "s_branch L_end" PH "_%=\n\t"

// The first blocks of a programme are the request blocks of chunks 0 and 1 (2 blocks; 4 with centres and curvatures).
#define A2R_FIRST_PLAIN(TB)                                                                                         \
    "s_load_dwordx16 s[36:51], %[prog], 0x0\n\t"                                                                    \
    "s_load_dwordx16 s[52:67], %[prog], 0x40\n\t"                                                                   \
    "s_load_dwordx16 s[68:83], %[prog], 0x80\n\t"                                                                   \
    "s_load_dwordx16 s[84:99], %[prog], 0xc0\n\t"                                                                   \
    "s_waitcnt lgkmcnt(0)\n\t"                                                                                      \
    A2R_REQ_PLAIN(TB, "0", "40", "0", "0") A2R_REQ_PLAIN(TB, "8", "72", "0", "0")                                   \
    "s_mov_b32 s26, 0x100\n\t"
#define A2R_FIRST_TWO(TB, REQ)                                                                                      \
    "s_load_dwordx16 s[36:51], %[prog], 0x0\n\t"                                                                    \
    "s_load_dwordx16 s[52:67], %[prog], 0x40\n\t"                                                                   \
    "s_load_dwordx16 s[68:83], %[prog], 0x80\n\t"                                                                   \
    "s_load_dwordx16 s[84:99], %[prog], 0xc0\n\t"                                                                   \
    "s_waitcnt lgkmcnt(0)\n\t"                                                                                      \
    REQ(TB, "0", "40", "68", "84")                                                                                  \
    "s_load_dwordx16 s[36:51], %[prog], 0x100\n\t"                                                                  \
    "s_load_dwordx16 s[52:67], %[prog], 0x140\n\t"                                                                  \
    "s_load_dwordx16 s[68:83], %[prog], 0x180\n\t"                                                                  \
    "s_load_dwordx16 s[84:99], %[prog], 0x1c0\n\t"                                                                  \
    "s_waitcnt lgkmcnt(0)\n\t"                                                                                      \
    REQ(TB, "8", "40", "68", "84")                                                                                  \
    "s_mov_b32 s26, 0x200\n\t"
#define A2R_FIRST_FULL(TB) A2R_FIRST_TWO(TB, A2R_REQ_FULL)
#define A2R_FIRST_HC(TB) A2R_FIRST_TWO(TB, A2R_REQ_HC)

// s26: byte offset of the next block to fetch.  Block A is fetched while block B is being applied and the other
// way round; scalar loads return in no fixed order, so the wait for a block comes before the next fetch is issued.
// VARIANT: PLAIN, HC or FULL (pasted into macro names).
#define A2R_PROGRAMME(TB, GOSSIP, GRAD, AT, VARIANT)                                                                \
    A2R_ROWS(A2R_LD1)                                                                                               \
    "s_mov_b32 s28, 0\n\t"                                                                                          \
    "s_mov_b32 s29, 0\n\t"                                                                                          \
    "s_mov_b32 s30, 0\n\t"                                                                                          \
    A2R_FIRST_##VARIANT(TB)                                                                                         \
    "s_waitcnt vmcnt(0)\n\t"                                                                                        \
    "s_cmp_lt_u32 s26, %[nbytes]\n\t"                                                                               \
    "s_cbranch_scc0 L_end_%=\n\t"                                                                                   \
    "s_load_dwordx16 s[36:51], %[prog], s26\n\t"                                                                    \
    "s_add_u32 s27, s26, 64\n\t"                                                                                    \
    "s_load_dwordx16 s[52:67], %[prog], s27\n\t"                                                                    \
    "s_add_u32 s26, s26, 128\n"                                                                                     \
    "L_blka_%=:\n\t"                                                                                                \
    "s_waitcnt lgkmcnt(0)\n\t"                                                                                      \
    "s_cmp_lt_u32 s26, %[nbytes]\n\t"                                                                               \
    "s_cbranch_scc0 L_nob_%=\n\t"                                                                                   \
    "s_load_dwordx16 s[68:83], %[prog], s26\n\t"                                                                    \
    "s_add_u32 s27, s26, 64\n\t"                                                                                    \
    "s_load_dwordx16 s[84:99], %[prog], s27\n"                                                                      \
    "L_nob_%=:\n\t"                                                                                                 \
    "s_add_u32 s26, s26, 128\n\t"                                                                                   \
    A2R_SKIP_TEST_##VARIANT("a")                                                                                    \
    A2R_SLOTS_A(A2R_SLOT, A2R_SLOT, TB, GOSSIP)                                                                     \
    "\nL_enda_%=:\n\t"                                                                                              \
    "s_cmp_le_u32 s26, %[nbytes]\n\t"                                                                               \
    "s_cbranch_scc0 L_end_%=\n\t"                                                                                   \
    "s_waitcnt lgkmcnt(0)\n\t"                                                                                      \
    "s_cmp_lt_u32 s26, %[nbytes]\n\t"                                                                               \
    "s_cbranch_scc0 L_noa_%=\n\t"                                                                                   \
    "s_load_dwordx16 s[36:51], %[prog], s26\n\t"                                                                    \
    "s_add_u32 s27, s26, 64\n\t"                                                                                    \
    "s_load_dwordx16 s[52:67], %[prog], s27\n"                                                                      \
    "L_noa_%=:\n\t"                                                                                                 \
    "s_add_u32 s26, s26, 128\n\t"                                                                                   \
    A2R_SKIP_TEST_##VARIANT("b")                                                                                    \
    A2R_SLOTS_B(A2R_SLOT, A2R_SLOT, TB, GOSSIP)                                                                     \
    "\nL_endb_%=:\n\t"                                                                                              \
    "s_cmp_le_u32 s26, %[nbytes]\n\t"                                                                               \
    "s_cbranch_scc1 L_blka_%=\n\t"                                                                                  \
    "s_branch L_end_%=\n\t"                                                                                         \
    A2R_SLOTS_A(A2R_OTHER_FIRST, A2R_OTHER, TB, GRAD, AT, "a")                                                      \
    A2R_SLOTS_B(A2R_OTHER_FIRST, A2R_OTHER, TB, GRAD, AT, "b")                                                      \
    A2R_SWITCH(TB, "a", A2R_REQ_##VARIANT, VARIANT, "40", "68", "84")                                               \
    A2R_SWITCH(TB, "b", A2R_REQ_##VARIANT, VARIANT, "72", "36", "52")                                               \
    "\nL_end_%=:\n\t"                                                                                               \
    A2R_OFF                                                                                                         \
    "s_waitcnt vmcnt(0) lgkmcnt(0)"

// The rows of the tile into the state registers and back, 64 unrolled steps with running row addresses in scalar
// registers (written in C++, the compiler forms all 128 row addresses first and parks them in spare vector lanes).
// s[40:41], s[42:43]: address of the current row of x and of xt (the lane adds the byte offset of its column); an untouched worker's registers
// are loaded from the first touched row (never used, never stored), so every register is defined.
#define A2R_LD1(b, k)                                                                                               \
    "s_bitcmp1_b64 %[touched], " #b "+" #k "\n\t"                                                                   \
    "s_cselect_b64 s[44:45], s[40:41], %[p0]\n\t"                                                                   \
    "s_cselect_b64 s[46:47], s[42:43], %[q0]\n\t"                                                                   \
    "global_load_dword v[" #b "+" #k "], %[voff], s[44:45] nt\n\t"                                                  \
    "global_load_dword v[64+" #b "+" #k "], %[voff], s[46:47] nt\n\t"                                               \
    "s_add_u32 s40, s40, %[slo]\n\t"                                                                                \
    "s_addc_u32 s41, s41, %[shi]\n\t"                                                                               \
    "s_add_u32 s42, s42, %[slo]\n\t"                                                                                \
    "s_addc_u32 s43, s43, %[shi]\n\t"
#define A2R_ST1(b, k)                                                                                               \
    "s_bitcmp1_b64 %[touched], " #b "+" #k "\n\t"                                                                   \
    "s_cbranch_scc0 L_st" #b "_" #k "_%=\n\t"                                                                       \
    "global_store_dword %[voff], v[" #b "+" #k "], s[40:41] nt\n\t"                                                 \
    "global_store_dword %[voff], v[64+" #b "+" #k "], s[42:43] nt\n"                                                \
    "L_st" #b "_" #k "_%=:\n\t"                                                                                     \
    "s_add_u32 s40, s40, %[slo]\n\t"                                                                                \
    "s_addc_u32 s41, s41, %[shi]\n\t"                                                                               \
    "s_add_u32 s42, s42, %[slo]\n\t"                                                                                \
    "s_addc_u32 s43, s43, %[shi]\n\t"
#define A2R_ROWS8(M, b) M(b, 0) M(b, 1) M(b, 2) M(b, 3) M(b, 4) M(b, 5) M(b, 6) M(b, 7)
#define A2R_ROWS(M)                                                                                                 \
    "s_mov_b64 s[40:41], %[xb]\n\t"                                                                                 \
    "s_mov_b64 s[42:43], %[tb]\n\t"                                                                                 \
    A2R_ROWS8(M, 0) A2R_ROWS8(M, 8) A2R_ROWS8(M, 16) A2R_ROWS8(M, 24)                                               \
    A2R_ROWS8(M, 32) A2R_ROWS8(M, 40) A2R_ROWS8(M, 48) A2R_ROWS8(M, 56)

#define A2R_S10(a) "s" #a "0", "s" #a "1", "s" #a "2", "s" #a "3", "s" #a "4", "s" #a "5", "s" #a "6", "s" #a "7", "s" #a "8", "s" #a "9"
#define A2R_CLOBBER_S "s26", "s27", "s28", "s29", "s30", "s31", "s36", "s37", "s38", "s39", A2R_S10(4), A2R_S10(5), A2R_S10(6), A2R_S10(7), A2R_S10(8), A2R_S10(9), "vcc", "scc", "memory"
#define A2R_V10(a) "v" #a "0", "v" #a "1", "v" #a "2", "v" #a "3", "v" #a "4", "v" #a "5", "v" #a "6", "v" #a "7", "v" #a "8", "v" #a "9"
#define A2R_CLOBBER_PLAIN "v128", "v129", A2R_V10(13), A2R_V10(14), "v150"
#define A2R_CLOBBER_HC "v128", "v129", A2R_V10(13), A2R_V10(14), A2R_V10(15), "v160", "v161", "v162", "v163", "v164", "v165", "v166"
#define A2R_CLOBBER_FULL                                                                                            \
    "v128", "v129", A2R_V10(13), A2R_V10(14), A2R_V10(15), A2R_V10(16), A2R_V10(17), "v180", "v181", "v182"

// VARIANT: 0 no centres and no curvatures, 1 centres only, 2 both.
template <bool PRE, int VARIANT>
__global__ __launch_bounds__(64) void regfile_kernel(float *__restrict__ x, float *__restrict__ xt, int64_t ld,
                                                     int64_t d, const ResSlot *__restrict__ recs, uint32_t n_bytes,
                                                     uint64_t touched, float alpha, float alpha_t) {
    const uint32_t lane = threadIdx.x;
    const int64_t col0 = (int64_t)blockIdx.x * 64;
    const bool valid = col0 + lane < d;
    const uint32_t lane_in = valid ? lane : 0u;             // loads of lanes past the end read the tile's first column
    const uint32_t voff = (uint32_t)(col0 + lane_in) * 4u;  // byte offset of the lane's column in a row (d <= 2^29)

    // The statement below loads the rows of the tile (A2R_ROWS), issues the first requests of gradient inputs, waits
    // for all of it and runs the programme; the four values it defines are the state registers.
    v32f X0, X1, T0, T1;
    const uintptr_t xb = reg_uniform(x), tb = reg_uniform(xt);     // the lane's offset counts from the start of a row
    const uint64_t step = (uint64_t)ld * 4u;
    const uint32_t step_lo = (uint32_t)step, step_hi = (uint32_t)(step >> 32);
    const uint64_t first = (uint64_t)(touched ? __builtin_ctzll(touched) : 0) * step;
    const uintptr_t p0 = xb + first, q0 = tb + first;
    const float neg_alpha = -alpha, neg_alpha_t = -alpha_t;
#define A2R_OPERANDS                                                                                                \
    : "=&{v[0:31]}"(X0), "=&{v[32:63]}"(X1), "=&{v[64:95]}"(T0), "=&{v[96:127]}"(T1)                                \
    : [prog] "s"(recs), [nbytes] "s"(n_bytes), [voff] "v"(voff),                                                    \
      [al] "s"(alpha), [nal] "s"(neg_alpha), [alt] "s"(alpha_t), [nalt] "s"(neg_alpha_t),                           \
      [xb] "s"(xb), [tb] "s"(tb), [p0] "s"(p0), [q0] "s"(q0), [slo] "s"(step_lo), [shi] "s"(step_hi),               \
      [touched] "s"(touched)
    if constexpr (VARIANT == 0) {
        if constexpr (!PRE)
            asm volatile(A2R_PROGRAMME("144", A2R_GOSSIP_0, A2R_GRAD_PLAIN, 2, PLAIN) A2R_OPERANDS
                         : A2R_CLOBBER_S, A2R_CLOBBER_PLAIN);
        else
            asm volatile(A2R_PROGRAMME("144", A2R_GOSSIP_1, A2R_GRAD_PLAIN, 4, PLAIN) A2R_OPERANDS
                         : A2R_CLOBBER_S, A2R_CLOBBER_PLAIN);
    } else if constexpr (VARIANT == 1) {
        if constexpr (!PRE)
            asm volatile(A2R_PROGRAMME("160", A2R_GOSSIP_0, A2R_GRAD_HC, 2, HC) A2R_OPERANDS
                         : A2R_CLOBBER_S, A2R_CLOBBER_HC);
        else
            asm volatile(A2R_PROGRAMME("160", A2R_GOSSIP_1, A2R_GRAD_HC, 4, HC) A2R_OPERANDS
                         : A2R_CLOBBER_S, A2R_CLOBBER_HC);
    } else {
        if constexpr (!PRE)
            asm volatile(A2R_PROGRAMME("176", A2R_GOSSIP_0, A2R_GRAD_FULL, 2, FULL) A2R_OPERANDS
                         : A2R_CLOBBER_S, A2R_CLOBBER_FULL);
        else
            asm volatile(A2R_PROGRAMME("176", A2R_GOSSIP_1, A2R_GRAD_FULL, 4, FULL) A2R_OPERANDS
                         : A2R_CLOBBER_S, A2R_CLOBBER_FULL);
    }
#undef A2R_OPERANDS

    if (valid) {
        asm volatile(A2R_ROWS(A2R_ST1)
                     :
                     : "{v[0:31]}"(X0), "{v[32:63]}"(X1), "{v[64:95]}"(T0), "{v[96:127]}"(T1), [xb] "s"(xb), [tb] "s"(tb),
                       [slo] "s"(step_lo), [shi] "s"(step_hi), [touched] "s"(touched), [voff] "v"(voff)
                     : "s40", "s41", "s42", "s43", "scc", "memory");
    }
}

// ------------------------------------------------------------------------------------------
// Plain device copy of n4 float4 pieces with the event kernels' access shape (4 pieces per lane,
// 256 lanes, non-temporal).  A measurement aid: it moves a known number of bytes, which gives
// the practical streaming ceiling of the machine at hand and the scale of the HBM counters.
// ------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void copy_probe_kernel(const v4f *__restrict__ src, v4f *__restrict__ dst,
                                                         int64_t n4) {
    const int64_t base = (int64_t)blockIdx.x * 1024 + threadIdx.x;
    v4f r[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
        const int64_t k = base + u * 256;
        if (k < n4) r[u] = __builtin_nontemporal_load(src + k);
    }
#pragma unroll
    for (int u = 0; u < 4; ++u) {
        const int64_t k = base + u * 256;
        if (k < n4) __builtin_nontemporal_store(r[u], dst + k);
    }
}

// ------------------------------------------------------------------------------------------
// In-place streaming probe with the walk kernel's access shape: grid = column tiles of TPB float4 pieces; every
// workgroup makes n_ops passes, pass k reading ROWS consecutive workers' pieces of x and xt (2 ROWS loads of 16
// bytes per lane, all issued before the first use), multiplying them by `scale` and storing them back in place
// (ordinary, temporal accesses).  The workers advance cyclically by ROWS per pass, so a row comes back after
// n / ROWS passes: with 64 workers and thousands of resident workgroups that is hundreds of megabytes later, beyond
// every cache of the chip, which makes the probe's rate the machine's in-place HBM streaming rate at this shape.
// ROWS = 2 is the shape of a gossip event (4 row pieces in, 4 out), ROWS = 1 that of a gradient event without
// inputs or of a pure mixing pass.  With scale = 1 the state is unchanged bit for bit (the host passes it at run
// time, so the arithmetic cannot be folded away).  Moves n_ops * ROWS * 64 bytes per whole float4 column.
// ------------------------------------------------------------------------------------------
template <int ROWS, int TPB>
__global__ __launch_bounds__(TPB) void inplace_probe_kernel(float *__restrict__ x, float *__restrict__ xt, int64_t ld,
                                                            int64_t d, int32_t n, int32_t n_ops, float scale) {
    const int64_t k = (int64_t)blockIdx.x * TPB + threadIdx.x;
    if (k >= (d >> 2)) return;
    const int64_t ld4 = ld >> 2;
    v4f *const px = (v4f *)x + k, *const pxt = (v4f *)xt + k;
    int32_t w = 0;
    for (int32_t op = 0; op < n_ops; ++op) {
        v4f a[ROWS], at[ROWS];
        int32_t row[ROWS];
#pragma unroll
        for (int r = 0; r < ROWS; ++r) {
            row[r] = w + r < n ? w + r : w + r - n;
            a[r] = px[(int64_t)row[r] * ld4];
            at[r] = pxt[(int64_t)row[r] * ld4];
        }
#pragma unroll
        for (int r = 0; r < ROWS; ++r) {
            px[(int64_t)row[r] * ld4] = a[r] * scale;
            pxt[(int64_t)row[r] * ld4] = at[r] * scale;
        }
        w = w + ROWS < n ? w + ROWS : w + ROWS - n;
    }
}

// ------------------------------------------------------------------------------------------
// Observables.  One pass over x and xt (8 n d bytes).  A workgroup owns tiles of
// V * 256 float4 columns and walks all n rows of a tile, so that for every column it sees the
// n workers' values and can form the column's contribution to ||pi x||_F^2 without a second
// pass: with the first row's (mixed) value p as pivot, D_i = v_i - p in fp64,
//     sum_i (v_i - mean)^2 = sum_i D_i^2 - (sum_i D_i)^2 / n.
// The pending mixing of each worker up to the observation time is applied in registers from
// a per-worker coefficient table staged in LDS; nothing is written back to x or xt.
// Per-worker coordinate sums: fp32 partial over the 4 V columns of a lane and the 64 lanes of
// a wave (one partial = 256 V columns), then fp64 accumulation per wave in LDS.
// Output: partials[block][0..n) row sums of x, [n..2n) of xt, [2n] consensus x, [2n+1] xt.
// Dynamic LDS: kWaves * 2n doubles + n floats.
// ------------------------------------------------------------------------------------------
__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
    return v;
}

__device__ __forceinline__ v4f load4_guarded(const float *row, int64_t g, int64_t d) {
    // float4 piece g of a row of d valid floats; pieces or components past the end read as 0
    const int64_t k = g << 2;
    if (k + 4 <= d) return *(const v4f *)(row + k);
    v4f v = {0.f, 0.f, 0.f, 0.f};
    if (k < d) v.x = row[k];
    if (k + 1 < d) v.y = row[k + 1];
    if (k + 2 < d) v.z = row[k + 2];
    return v;
}

// Column accumulators of one lane: sum and sum of squares of the pivot-shifted values.
template <int V>
struct ColumnAcc {
    v4f px[V], pxt[V];
    double sx[V][4], qx[V][4], sxt[V][4], qxt[V][4];
};

// One row of a tile: mix, per-row partial sums into the wave's LDS slab, column accumulators.
template <int V>
__device__ __forceinline__ void stats_row(ColumnAcc<V> &acc, v4f (&a)[V], v4f (&at)[V], float b, bool first,
                                          double *my_row, int32_t i, int32_t n, int lane) {
    float rx = 0.f, rxt = 0.f;
#pragma unroll
    for (int u = 0; u < V; ++u) {
        mix(a[u], at[u], b);
        rx += (a[u].x + a[u].y) + (a[u].z + a[u].w);
        rxt += (at[u].x + at[u].y) + (at[u].z + at[u].w);
        if (first) { acc.px[u] = a[u]; acc.pxt[u] = at[u]; }
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            const double dx = (double)a[u][c] - (double)acc.px[u][c];
            const double dxt = (double)at[u][c] - (double)acc.pxt[u][c];
            acc.sx[u][c] += dx; acc.qx[u][c] += dx * dx;
            acc.sxt[u][c] += dxt; acc.qxt[u][c] += dxt * dxt;
        }
    }
    rx = wave_sum(rx);
    rxt = wave_sum(rxt);
    if (lane == 0) { my_row[i] += (double)rx; my_row[n + i] += (double)rxt; }
}

// Where the observables kernel finds the pending mixing coefficient of each worker: a device table (NULL: nothing
// is pending, every coefficient is 0) or the kernel's own argument block (no upload, nothing to keep alive).
struct MixTable {
    const float *p;
    __device__ __forceinline__ float at(int i) const { return p ? p[i] : 0.f; }
};
constexpr int kMixArgsMax = 256;         // workers whose coefficients fit into the argument block (1 KiB)
struct MixArgs {
    float b[kMixArgsMax];
    __device__ __forceinline__ float at(int i) const { return b[i]; }
};

// V: float4 pieces per lane and row; R: rows whose loads are issued together (memory-level parallelism).
template <int V, int R, bool NT, typename B>
__device__ __forceinline__ void stats_body(const float *__restrict__ x, const float *__restrict__ xt, int64_t ld,
                                           int64_t d, int32_t n, const B &bmix, double *__restrict__ partials,
                                           int64_t n_tiles) {
    extern __shared__ double smem[];
    double *srow = smem;                                  // [kWaves][2n]
    float *sb = (float *)(smem + (size_t)kWaves * 2 * n); // [n]
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    for (int i = tid; i < n; i += kThreads) sb[i] = bmix.at(i);
    for (int i = tid; i < kWaves * 2 * n; i += kThreads) srow[i] = 0.0;
    __syncthreads();
    double *my_row = srow + (size_t)wave * 2 * n;
    const double inv_n = 1.0 / (double)n;
    const int64_t n4 = d >> 2;
    double cons_x = 0.0, cons_xt = 0.0;

    for (int64_t tile = blockIdx.x; tile < n_tiles; tile += gridDim.x) {
        const int64_t g0 = tile * (V * kThreads) + tid;
        const bool full = (tile + 1) * (V * kThreads) <= n4;   // every piece of the tile is a whole float4
        ColumnAcc<V> acc;
#pragma unroll
        for (int u = 0; u < V; ++u)
#pragma unroll
            for (int c = 0; c < 4; ++c) acc.sx[u][c] = acc.qx[u][c] = acc.sxt[u][c] = acc.qxt[u][c] = 0.0;

        int32_t i = 0;
        if (full) {
            for (; i + R <= n; i += R) {
                v4f a[R][V], at[R][V];
#pragma unroll
                for (int r = 0; r < R; ++r) {
                    const v4f *xr = (const v4f *)(x + (int64_t)(i + r) * ld) + g0;
                    const v4f *xtr = (const v4f *)(xt + (int64_t)(i + r) * ld) + g0;
#pragma unroll
                    for (int u = 0; u < V; ++u) { a[r][u] = load4<NT>(xr + u * kThreads); at[r][u] = load4<NT>(xtr + u * kThreads); }
                }
#pragma unroll
                for (int r = 0; r < R; ++r)
                    stats_row<V>(acc, a[r], at[r], sb[i + r], i + r == 0, my_row, i + r, n, lane);
            }
        }
        for (; i < n; ++i) {
            const float *xr = x + (int64_t)i * ld, *xtr = xt + (int64_t)i * ld;
            v4f a[V], at[V];
#pragma unroll
            for (int u = 0; u < V; ++u) {
                a[u] = load4_guarded(xr, g0 + u * kThreads, d);
                at[u] = load4_guarded(xtr, g0 + u * kThreads, d);
            }
            stats_row<V>(acc, a, at, sb[i], i == 0, my_row, i, n, lane);
        }
#pragma unroll
        for (int u = 0; u < V; ++u)
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                cons_x += acc.qx[u][c] - acc.sx[u][c] * acc.sx[u][c] * inv_n;
                cons_xt += acc.qxt[u][c] - acc.sxt[u][c] * acc.sxt[u][c] * inv_n;
            }
    }

    // workgroup reduction of the two consensus partials (fixed order -> deterministic)
    __shared__ double scons[2][kThreads];
    scons[0][tid] = cons_x;
    scons[1][tid] = cons_xt;
    __syncthreads();
    for (int s = kThreads / 2; s > 0; s >>= 1) {
        if (tid < s) { scons[0][tid] += scons[0][tid + s]; scons[1][tid] += scons[1][tid + s]; }
        __syncthreads();
    }
    double *out = partials + (size_t)blockIdx.x * (2 * (size_t)n + 2);
    for (int i = tid; i < 2 * n; i += kThreads) {
        double s = 0.0;
#pragma unroll
        for (int w = 0; w < kWaves; ++w) s += srow[(size_t)w * 2 * n + i];
        out[i] = s;
    }
    if (tid == 0) { out[2 * n] = scons[0][0]; out[2 * n + 1] = scons[1][0]; }
}

template <int V, int R, bool NT>
__global__ __launch_bounds__(kThreads) void stats_kernel(const float *__restrict__ x,
                                                         const float *__restrict__ xt,
                                                         int64_t ld, int64_t d, int32_t n,
                                                         const float *__restrict__ bmix,
                                                         double *__restrict__ partials,
                                                         int64_t n_tiles) {
    stats_body<V, R, NT>(x, xt, ld, d, n, MixTable{bmix}, partials, n_tiles);
}

// The same pass with the coefficients in the argument block (n <= kMixArgsMax).
template <int V, int R, bool NT>
__global__ __launch_bounds__(kThreads) void stats_args_kernel(const float *__restrict__ x,
                                                              const float *__restrict__ xt,
                                                              int64_t ld, int64_t d, int32_t n,
                                                              const MixArgs bmix,
                                                              double *__restrict__ partials,
                                                              int64_t n_tiles) {
    stats_body<V, R, NT>(x, xt, ld, d, n, bmix, partials, n_tiles);
}

// Consensus step: every worker's (virtually mixed) row is replaced by the mean over workers, in x and in xt.
// One pass: a lane reads its float4 of all n rows (fp64 column sums), then writes the mean n times.
// 8 n d bytes in, 8 n d bytes out.  Dynamic LDS: n floats (pending mixing coefficients).
__global__ __launch_bounds__(kThreads) void average_kernel(float *__restrict__ x, float *__restrict__ xt,
                                                           int64_t ld, int64_t d, int32_t n,
                                                           const float *__restrict__ bmix) {
    extern __shared__ float sbm[];
    for (int i = threadIdx.x; i < n; i += kThreads) sbm[i] = bmix[i];
    __syncthreads();
    const int64_t g = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    const int64_t k = g << 2;
    if (k >= d) return;
    const bool whole = k + 4 <= d;
    double sx[4] = {0.0, 0.0, 0.0, 0.0}, sxt[4] = {0.0, 0.0, 0.0, 0.0};
    for (int32_t i = 0; i < n; ++i) {
        v4f a = load4_guarded(x + (int64_t)i * ld, g, d), at = load4_guarded(xt + (int64_t)i * ld, g, d);
        mix(a, at, sbm[i]);
#pragma unroll
        for (int c = 0; c < 4; ++c) { sx[c] += (double)a[c]; sxt[c] += (double)at[c]; }
    }
    v4f mx, mxt;
#pragma unroll
    for (int c = 0; c < 4; ++c) { mx[c] = (float)(sx[c] / (double)n); mxt[c] = (float)(sxt[c] / (double)n); }
    for (int32_t i = 0; i < n; ++i) {
        float *xr = x + (int64_t)i * ld + k, *xtr = xt + (int64_t)i * ld + k;
        if (whole) { *(v4f *)xr = mx; *(v4f *)xtr = mxt; }
        else for (int c = 0; c < 4 && k + c < d; ++c) { xr[c] = mx[c]; xtr[c] = mxt[c]; }
    }
}

// Sums the per-workgroup partials: workgroup j produces out[j] = sum_b partials[b][j].  Lane t adds
// blocks t, t + 256, ... in order, then a fixed-shape tree combines the 256 lanes (deterministic).
__global__ __launch_bounds__(kThreads) void stats_final_kernel(const double *__restrict__ partials,
                                                               int32_t n_blocks, int32_t m,
                                                               double *__restrict__ out) {
    __shared__ double acc[kThreads];
    const int j = blockIdx.x, tid = threadIdx.x;
    double s = 0.0;
    for (int32_t b = tid; b < n_blocks; b += kThreads) s += partials[(size_t)b * m + j];
    acc[tid] = s;
    __syncthreads();
    for (int w = kThreads / 2; w > 0; w >>= 1) {
        if (tid < w) acc[tid] += acc[tid + w];
        __syncthreads();
    }
    if (tid == 0) out[j] = acc[0];
}

}  // namespace a2cid
