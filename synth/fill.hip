// Device side of the shared synthetic-input generator (see synth/gen.py for the definition).
// Harness code: fills device buffers with the seeded fp32 Gaussian stream so that initial
// states, c_i and per-event gradient noise never have to cross PCIe.  It performs none of the
// method's arithmetic and is not part of liba2cid.so.
//
// Bit-exactness with the numpy implementation requires individually rounded fp32 operations:
// this file must be compiled with -ffp-contract=off and without fast-math.
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace {

typedef float v4f __attribute__((ext_vector_type(4)));

__device__ __forceinline__ void philox4x32_10(uint32_t &c0, uint32_t &c1, uint32_t &c2, uint32_t &c3,
                                              uint32_t k0, uint32_t k1) {
#pragma unroll
    for (int r = 0; r < 10; ++r) {
        const uint32_t h0 = __umulhi(0xD2511F53u, c0), l0 = 0xD2511F53u * c0;
        const uint32_t h1 = __umulhi(0xCD9E8D57u, c2), l1 = 0xCD9E8D57u * c2;
        const uint32_t n0 = h1 ^ c1 ^ k0, n2 = h0 ^ c3 ^ k1;
        c0 = n0; c1 = l1; c2 = n2; c3 = l0;
        k0 += 0x9E3779B9u; k1 += 0xBB67AE85u;
    }
}

__device__ __forceinline__ void box_muller(uint32_t w0, uint32_t w1, float &z0, float &z1) {
    const float u1 = ((float)(w0 >> 9) + 0.5f) * 0x1.0p-23f;
    const uint32_t bits = __float_as_uint(u1);
    int e = (int)(bits >> 23) - 127;
    float m = __uint_as_float((bits & 0x007FFFFFu) | 0x3F800000u);
    if (m > 1.41421353816986083984375f) { m = m * 0.5f; e += 1; }
    const float s = (m - 1.0f) / (m + 1.0f);
    const float z = s * s;
    float p = 0x1.c71c72p-4f * z + 0x1.24924ap-3f;   // 1/9, 1/7 rounded to fp32
    p = p * z + 0x1.99999ap-3f;                        // 1/5
    p = p * z + 0x1.555556p-2f;                        // 1/3
    p = p * z + 1.0f;
    const float ln = (float)e * 0.693147182464599609375f + (s + s) * p;
    const float neg = -ln;
    const float r = sqrtf(neg + neg);   // correctly rounded (the _rn intrinsic is not)

    const uint32_t w = w1 >> 8;
    const uint32_t quad = w >> 22;
    uint32_t fr = w & 0x3FFFFFu;
    const bool swap = fr > 0x200000u;
    if (swap) fr = 0x400000u - fr;
    const float phi = (float)fr * 0x1.921fb6p-22f;      // (pi/2) * 2^-22 rounded to fp32
    const float y = phi * phi;
    float ps = 0x1.71de3ap-19f * y + -0x1.a01a02p-13f;  // 1/9!, -1/7!
    ps = ps * y + 0x1.111112p-7f;                       // 1/5!
    ps = ps * y + -0x1.555556p-3f;                      // -1/3!
    ps = ps * y + 1.0f;
    float sn = phi * ps;
    float pc = -0x1.27e4fcp-22f * y + 0x1.a01a02p-16f;  // -1/10!, 1/8!
    pc = pc * y + -0x1.6c16c2p-10f;                     // -1/6!
    pc = pc * y + 0x1.555556p-5f;                       // 1/4!
    pc = pc * y + -0.5f;
    float cs = pc * y + 1.0f;
    if (swap) { const float tmp = sn; sn = cs; cs = tmp; }
    float co, so;
    switch (quad) {
        case 0: co = cs; so = sn; break;
        case 1: co = -sn; so = cs; break;
        case 2: co = -cs; so = -sn; break;
        default: co = sn; so = -cs; break;
    }
    z0 = r * co;
    z1 = r * so;
}

__global__ __launch_bounds__(256) void fill_normal_kernel(float *out, int64_t d, uint32_t seed_lo, uint32_t seed_hi,
                                                          uint32_t domain, uint32_t row_lo, uint32_t row_hi,
                                                          float sigma, float mean) {
    const int64_t groups = (d + 3) >> 2;
    for (int64_t q = (int64_t)blockIdx.x * 256 + threadIdx.x; q < groups; q += (int64_t)gridDim.x * 256) {
        uint32_t c0 = (uint32_t)q, c1 = row_lo, c2 = row_hi, c3 = domain;
        philox4x32_10(c0, c1, c2, c3, seed_lo, seed_hi);
        float z[4];
        box_muller(c0, c1, z[0], z[1]);
        box_muller(c2, c3, z[2], z[3]);
#pragma unroll
        for (int k = 0; k < 4; ++k) z[k] = mean + sigma * z[k];
        const int64_t col = q << 2;
        if (col + 4 <= d) {
            *(v4f *)(out + col) = (v4f){z[0], z[1], z[2], z[3]};
        } else {
            for (int k = 0; k < 4 && col + k < d; ++k) out[col + k] = z[k];
        }
    }
}

}  // namespace

// out: device pointer to d floats, 16-byte aligned.  Enqueues on `stream`; returns the HIP error code.
extern "C" int synth_fill_normal(float *out, int64_t d, uint64_t seed, uint32_t domain, uint64_t row,
                                 float sigma, float mean, void *stream) {
    if (!out || d < 1 || ((uintptr_t)out & 15u)) return -1;
    const int64_t groups = (d + 3) >> 2;
    int64_t blocks = (groups + 255) / 256;
    if (blocks > 8192) blocks = 8192;
    hipLaunchKernelGGL(fill_normal_kernel, dim3((unsigned)blocks), dim3(256), 0, (hipStream_t)stream, out, d,
                       (uint32_t)seed, (uint32_t)(seed >> 32), domain, (uint32_t)row, (uint32_t)(row >> 32),
                       sigma, mean);
    return (int)hipGetLastError();
}
