// Random augmentation (Transformations section: a random rotation and a random
// translation of at most a given distance, drawn per example).  The paper names
// neither a generator nor a distribution; this library draws
//   - from Philox4x32-10 (Salmon, Moraes, Dror, Shaw, SC'11): key = the 64-bit
//     seed, counter = (example b, the 64-bit draw number, block), block 0 for the
//     rotation and 1 for the translation, so example b's transform depends on
//     (seed, draw, b) alone and any subset of examples can be drawn anywhere;
//   - a rotation uniform over SO(3) by Shoemake's construction ("Uniform random
//     rotations", Graphics Gems III) from three uniforms;
//   - a translation uniform in [-T, T] on each axis.
// A word w becomes u = (w + 0.5) / 2^32, and everything up to the final rounding
// to float is double: B is small, and the drawn floats then do not depend on the
// float rounding of an intermediate.  One thread per example.
#include "mg_common.h"

namespace mg {

namespace {

struct Words {
    uint32_t w[4];
};

__device__ inline Words philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3,
                                      uint32_t k0, uint32_t k1)
{
    constexpr uint32_t kMul0 = 0xD2511F53u, kMul1 = 0xCD9E8D57u;       // round multipliers
    constexpr uint32_t kWeyl0 = 0x9E3779B9u, kWeyl1 = 0xBB67AE85u;     // key increments
#pragma unroll
    for (int round = 0; round < 10; ++round) {
        const uint32_t hi0 = __umulhi(kMul0, c0), lo0 = kMul0 * c0;
        const uint32_t hi1 = __umulhi(kMul1, c2), lo1 = kMul1 * c2;
        c0 = hi1 ^ c1 ^ k0;
        c1 = lo1;
        c2 = hi0 ^ c3 ^ k1;
        c3 = lo0;
        k0 += kWeyl0;
        k1 += kWeyl1;
    }
    Words o;
    o.w[0] = c0; o.w[1] = c1; o.w[2] = c2; o.w[3] = c3;
    return o;
}

__device__ inline double uniform01(uint32_t w) { return ((double)w + 0.5) * (1.0 / 4294967296.0); }

__global__ __launch_bounds__(64) void draw_kernel(uint32_t seed_lo, uint32_t seed_hi,
                                                  uint32_t draw_lo, uint32_t draw_hi, int B,
                                                  int random_rotation, double max_translation,
                                                  float *quats, float *translations)
{
    const int b = blockIdx.x * blockDim.x + threadIdx.x;
    if (b >= B) return;
    float q[4] = {1.0f, 0.0f, 0.0f, 0.0f}, t[3] = {0.0f, 0.0f, 0.0f};
    if (random_rotation) {
        const Words r = philox4x32_10((uint32_t)b, draw_lo, draw_hi, 0u, seed_lo, seed_hi);
        const double two_pi = 6.283185307179586476925286766559;
        const double u0 = uniform01(r.w[0]);
        const double a1 = two_pi * uniform01(r.w[1]), a2 = two_pi * uniform01(r.w[2]);
        const double s1 = sqrt(1.0 - u0), s2 = sqrt(u0);
        q[0] = (float)(s2 * cos(a2));
        q[1] = (float)(s1 * sin(a1));
        q[2] = (float)(s1 * cos(a1));
        q[3] = (float)(s2 * sin(a2));
    }
    if (max_translation != 0.0) {
        const Words r = philox4x32_10((uint32_t)b, draw_lo, draw_hi, 1u, seed_lo, seed_hi);
#pragma unroll
        for (int m = 0; m < 3; ++m)
            t[m] = (float)(max_translation * (2.0 * uniform01(r.w[m]) - 1.0));
    }
#pragma unroll
    for (int m = 0; m < 4; ++m) quats[4 * (size_t)b + m] = q[m];
#pragma unroll
    for (int m = 0; m < 3; ++m) translations[3 * (size_t)b + m] = t[m];
}

}  // namespace

hipError_t launch_draw_transforms(uint64_t seed, uint64_t draw, int B, bool random_rotation,
                                  float max_translation, float *quats, float *translations,
                                  hipStream_t stream)
{
    hipLaunchKernelGGL(draw_kernel, dim3((B + 63) / 64), dim3(64), 0, stream, (uint32_t)seed,
                       (uint32_t)(seed >> 32), (uint32_t)draw, (uint32_t)(draw >> 32), B,
                       random_rotation ? 1 : 0, (double)max_translation, quats, translations);
    return hipGetLastError();
}

}  // namespace mg
