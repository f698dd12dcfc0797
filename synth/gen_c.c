/* Host side of the shared input generator in C: the same definition as synth/gen.py (see there),
 * for the cases where numpy is too slow (millions of events x thousands of columns).
 * Must be compiled with -ffp-contract=off and without fast-math: every fp32 operation below is
 * meant to round on its own, exactly as in the numpy and the device implementations. */
#include <math.h>
#include <stdint.h>
#include <string.h>

static void philox4x32_10(uint32_t c[4], uint32_t k0, uint32_t k1)
{
    for (int r = 0; r < 10; ++r) {
        const uint64_t p0 = (uint64_t)0xD2511F53u * c[0];
        const uint64_t p1 = (uint64_t)0xCD9E8D57u * c[2];
        const uint32_t a = (uint32_t)(p1 >> 32) ^ c[1] ^ k0;
        const uint32_t b = (uint32_t)(p0 >> 32) ^ c[3] ^ k1;
        c[0] = a; c[1] = (uint32_t)p1; c[2] = b; c[3] = (uint32_t)p0;
        k0 += 0x9E3779B9u; k1 += 0xBB67AE85u;
    }
}

static void box_muller(uint32_t w0, uint32_t w1, float *z0, float *z1)
{
    const float u1 = ((float)(w0 >> 9) + 0.5f) * 0x1.0p-23f;
    uint32_t bits; memcpy(&bits, &u1, 4);
    int e = (int)(bits >> 23) - 127;
    uint32_t mb = (bits & 0x007FFFFFu) | 0x3F800000u;
    float m; memcpy(&m, &mb, 4);
    if (m > 1.41421353816986083984375f) { m = m * 0.5f; e += 1; }
    const float s = (m - 1.0f) / (m + 1.0f);
    const float z = s * s;
    float p = 0x1.c71c72p-4f * z + 0x1.24924ap-3f;
    p = p * z + 0x1.99999ap-3f;
    p = p * z + 0x1.555556p-2f;
    p = p * z + 1.0f;
    const float ln = (float)e * 0.693147182464599609375f + (s + s) * p;
    const float neg = -ln;
    const float r = sqrtf(neg + neg);

    const uint32_t w = w1 >> 8;
    const uint32_t quad = w >> 22;
    uint32_t fr = w & 0x3FFFFFu;
    const int swap = fr > 0x200000u;
    if (swap) fr = 0x400000u - fr;
    const float phi = (float)fr * 0x1.921fb6p-22f;
    const float y = phi * phi;
    float ps = 0x1.71de3ap-19f * y + -0x1.a01a02p-13f;
    ps = ps * y + 0x1.111112p-7f;
    ps = ps * y + -0x1.555556p-3f;
    ps = ps * y + 1.0f;
    float sn = phi * ps;
    float pc = -0x1.27e4fcp-22f * y + 0x1.a01a02p-16f;
    pc = pc * y + -0x1.6c16c2p-10f;
    pc = pc * y + 0x1.555556p-5f;
    pc = pc * y + -0.5f;
    float cs = pc * y + 1.0f;
    if (swap) { const float t = sn; sn = cs; cs = t; }
    float co, so;
    switch (quad) {
        case 0: co = cs; so = sn; break;
        case 1: co = -sn; so = cs; break;
        case 2: co = -cs; so = -sn; break;
        default: co = sn; so = -cs; break;
    }
    *z0 = r * co;
    *z1 = r * so;
}

/* out[r * n_cols + k] = value(seed, domain, rows[r], cols[k]) */
void synth_normal_rows(uint64_t seed, uint32_t domain, const int64_t *rows, int64_t n_rows,
                       const int64_t *cols, int64_t n_cols, float sigma, float mean, float *out)
{
    for (int64_t r = 0; r < n_rows; ++r) {
        const uint64_t row = (uint64_t)rows[r];
        int64_t cached_q = -1;
        float z[4] = {0, 0, 0, 0};
        for (int64_t k = 0; k < n_cols; ++k) {
            const int64_t q = cols[k] >> 2;
            if (q != cached_q) {
                uint32_t c[4] = {(uint32_t)q, (uint32_t)row, (uint32_t)(row >> 32), domain};
                philox4x32_10(c, (uint32_t)seed, (uint32_t)(seed >> 32));
                box_muller(c[0], c[1], &z[0], &z[1]);
                box_muller(c[2], c[3], &z[2], &z[3]);
                cached_q = q;
            }
            out[r * n_cols + k] = mean + sigma * z[cols[k] & 3];
        }
    }
}
