// Step 1 and 2 of the path: per-example coordinate transform, radius lookup,
// bounding-box culling and channel binning.
//
// Transform (Transformations section of the paper): x' = R(q)(x - c) + c + t,
// q = (w,x,y,z) with (1,0,0,0) the identity.  The arithmetic is double in one
// fixed order (no fused multiply-add; the file is compiled with
// -ffp-contract=off) and the result is rounded once to float, so that the
// binary-occupancy decision downstream is reproducible bit for bit:
//   n  = ((w*w + x*x) + y*y) + z*z          s = 2/n   (n == 0: identity)
//   xs = x*s, ys = y*s, zs = z*s
//   R  = [ 1-(y*ys+z*zs)   x*ys-w*zs      x*zs+w*ys   ]
//        [ x*ys+w*zs       1-(x*xs+z*zs)  y*zs-w*xs   ]
//        [ x*zs-w*ys       y*zs+w*xs      1-(x*xs+y*ys) ]
//   x'_m = (((R_m0*u0 + R_m1*u1) + R_m2*u2) + c_m) + t_m,   u = x - c
//
// Culling is exact: the density is identically zero beyond c(grm)*r, so an
// atom whose cutoff cube misses the grid box contributes nothing.
#include "mg_common.h"

namespace mg {

namespace {

constexpr int kPrepThreads = 256;
constexpr int kListCap = 1024;      // matches staged in LDS per round

struct Xform {
    double R[9];
    double c[3];
    double t[3];
};

__device__ inline void load_xform(Xform &X, int b, const float *centers, const float *quats,
                                  const float *translations)
{
    double w = 1.0, x = 0.0, y = 0.0, z = 0.0;
    if (quats) {
        w = (double)quats[4 * b + 0];
        x = (double)quats[4 * b + 1];
        y = (double)quats[4 * b + 2];
        z = (double)quats[4 * b + 3];
    }
    const double n = ((w * w + x * x) + y * y) + z * z;
    if (!(n > 0.0) || !(n < 1.0e300)) {
        X.R[0] = 1.0; X.R[1] = 0.0; X.R[2] = 0.0;
        X.R[3] = 0.0; X.R[4] = 1.0; X.R[5] = 0.0;
        X.R[6] = 0.0; X.R[7] = 0.0; X.R[8] = 1.0;
    } else {
        const double s = 2.0 / n;
        const double xs = x * s, ys = y * s, zs = z * s;
        const double wx = w * xs, wy = w * ys, wz = w * zs;
        const double xx = x * xs, xy = x * ys, xz = x * zs;
        const double yy = y * ys, yz = y * zs, zz = z * zs;
        X.R[0] = 1.0 - (yy + zz); X.R[1] = xy - wz;         X.R[2] = xz + wy;
        X.R[3] = xy + wz;         X.R[4] = 1.0 - (xx + zz); X.R[5] = yz - wx;
        X.R[6] = xz - wy;         X.R[7] = yz + wx;         X.R[8] = 1.0 - (xx + yy);
    }
    for (int m = 0; m < 3; ++m) {
        X.c[m] = centers ? (double)centers[3 * b + m] : 0.0;
        X.t[m] = translations ? (double)translations[3 * b + m] : 0.0;
    }
}

__device__ inline void apply_xform(const Xform &X, const float *p, float *o)
{
    const double u0 = (double)p[0] - X.c[0];
    const double u1 = (double)p[1] - X.c[1];
    const double u2 = (double)p[2] - X.c[2];
    o[0] = (float)((((X.R[0] * u0 + X.R[1] * u1) + X.R[2] * u2) + X.c[0]) + X.t[0]);
    o[1] = (float)((((X.R[3] * u0 + X.R[4] * u1) + X.R[5] * u2) + X.c[1]) + X.t[1]);
    o[2] = (float)((((X.R[6] * u0 + X.R[7] * u1) + X.R[8] * u2) + X.c[2]) + X.t[2]);
}

__global__ __launch_bounds__(256) void transform_kernel(int B, int N, const float *coords,
                                                        const float *centers, const float *quats,
                                                        const float *translations, float *out)
{
    const int b = blockIdx.y;
    const int a = blockIdx.x * blockDim.x + threadIdx.x;
    if (a >= N) return;
    Xform X;
    load_xform(X, b, centers, quats, translations);
    const size_t k = ((size_t)b * N + a) * 3;
    float o[3];
    apply_xform(X, coords + k, o);
    out[k + 0] = o[0];
    out[k + 1] = o[1];
    out[k + 2] = o[2];
}

// Exclusive prefix sum of `v` over the 256 threads of the block; *total gets the sum.
__device__ inline int block_exclusive_scan(int v, int *s_wave, int *total)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    int incl = v;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        const int up = __shfl_up(incl, d, 64);
        if (lane >= d) incl += up;
    }
    if (lane == 63) s_wave[wave] = incl;
    __syncthreads();
    int base = 0, sum = 0;
    for (int w = 0; w < kPrepThreads / 64; ++w) {
        const int c = s_wave[w];
        if (w < wave) base += c;
        sum += c;
    }
    __syncthreads();
    *total = sum;
    return base + incl - v;
}

// One workgroup per (type t, example b) for index types; per example for
// vector types (every atom belongs to the single group).
template <bool VECTOR>
__global__ __launch_bounds__(256) void prep_kernel(GridSpec gs, Batch bt, Workspace ws,
                                                   float *gclear, float *wclear)
{
    __shared__ int s_list[kListCap];
    __shared__ int s_wave[8];

    const int b = blockIdx.y, t = blockIdx.x, tid = threadIdx.x;
    const int N = bt.N, T = bt.T;
    int n = N;
    if (bt.natoms) {
        n = bt.natoms[b];
        n = n < 0 ? 0 : (n > N ? N : n);
    }
    const int32_t *ty = VECTOR ? nullptr : bt.types + (size_t)b * N;

    // every thread owns a run of consecutive atoms: keeps the binning stable
    const int per = (n + kPrepThreads - 1) / kPrepThreads;
    const int a0 = min(n, tid * per), a1 = min(n, a0 + per);
    int less = 0, eq = 0;
    if (VECTOR) {
        eq = a1 - a0;
    } else {
        for (int a = a0; a < a1; ++a) {
            const int v = ty[a];
            less += (v >= 0 && v < t) ? 1 : 0;
            eq += (v == t) ? 1 : 0;
        }
    }
    int M, first;
    const int my_first = block_exclusive_scan(eq, s_wave, &M);
    (void)block_exclusive_scan(less, s_wave, &first);
    if (VECTOR) first = 0;
    if (tid == 0) ws.meta[(size_t)b * T + t] = make_int2(first, M);

    Xform X;
    load_xform(X, b, bt.centers, bt.quats, bt.translations);
    if (t == 0 && tid < 9) ws.rot[b * 12 + tid] = (float)X.R[tid];

    // reach of the widest atom of this group, for vector types (radius per channel)
    float vec_reach = 0.0f;
    if (VECTOR) {
        for (int k = 0; k < T; ++k) {
            const float r = gs.radius_scale * bt.radii[k];
            if (r > vec_reach) vec_reach = r;
        }
        if (!gs.binary) vec_reach *= gs.c;
    }
    const float pad = 1.0e-3f * gs.res;
    const float span = (float)(gs.D - 1) * gs.res;
    float org[3];
    for (int m = 0; m < 3; ++m)
        org[m] = (bt.centers ? bt.centers[3 * b + m] : 0.0f) - gs.half;

    float4 *rec = ws.rec + (size_t)b * N + first;
    int *idx = ws.idx + (size_t)b * N + first;

    for (int r0 = 0; r0 < M; r0 += kListCap) {
        int rank = my_first;
        for (int a = a0; a < a1; ++a) {
            const bool match = VECTOR ? true : (ty[a] == t);
            if (match) {
                if (rank >= r0 && rank < r0 + kListCap) s_list[rank - r0] = a;
                ++rank;
            }
        }
        __syncthreads();
        const int cnt = min(kListCap, M - r0);
        for (int m = tid; m < cnt; m += kPrepThreads) {
            const int a = s_list[m];
            float p[3];
            apply_xform(X, bt.coords + ((size_t)b * N + a) * 3, p);
            float r, reach;
            if (VECTOR) {
                r = 1.0f;
                reach = vec_reach;
            } else {
                const float rad = gs.radius_type_indexed ? bt.radii[t] : bt.radii[(size_t)b * N + a];
                r = gs.radius_scale * rad;
                reach = gs.binary ? r : r * gs.c;
            }
            bool live = (r > 0.0f) && (reach < 1.0e30f);
            for (int k = 0; k < 3; ++k) {
                // also false for NaN / infinite coordinates
                live = live && (p[k] >= org[k] - reach - pad) && (p[k] <= org[k] + span + reach + pad);
            }
            rec[r0 + m] = make_float4(p[0], p[1], p[2], live ? r : 0.0f);
            idx[r0 + m] = a;
            if (!live) {
                if (gclear) {
                    float *g = gclear + ((size_t)b * N + a) * 3;
                    g[0] = 0.0f; g[1] = 0.0f; g[2] = 0.0f;
                }
                if (wclear)
                    for (int k = 0; k < T; ++k) wclear[((size_t)b * N + a) * T + k] = 0.0f;
            }
        }
        __syncthreads();
    }

    // atoms no group owns (past natoms, type outside [0,T)): zero gradients
    if (t == 0 && (gclear || wclear)) {
        for (int a = tid; a < N; a += kPrepThreads) {
            bool orphan = a >= n;
            if (!VECTOR && !orphan) {
                const int v = ty[a];
                orphan = v < 0 || v >= T;
            }
            if (!orphan) continue;
            if (gclear) {
                float *g = gclear + ((size_t)b * N + a) * 3;
                g[0] = 0.0f; g[1] = 0.0f; g[2] = 0.0f;
            }
            if (wclear)
                for (int k = 0; k < T; ++k) wclear[((size_t)b * N + a) * T + k] = 0.0f;
        }
    }
}

}  // namespace

size_t workspace_bytes(int B, int N, int T)
{
    const size_t bn = (size_t)B * (size_t)N;
    size_t bytes = bn * sizeof(float4);                         // rec
    bytes += ((bn * sizeof(int) + 15) / 16) * 16;               // idx
    bytes += (((size_t)B * T * sizeof(int2) + 15) / 16) * 16;   // meta
    bytes += (size_t)B * 12 * sizeof(float);                    // rot
    return bytes;
}

Workspace carve_workspace(void *base, int B, int N, int T)
{
    const size_t bn = (size_t)B * (size_t)N;
    char *p = (char *)base;
    Workspace ws;
    ws.rec = (float4 *)p;
    p += bn * sizeof(float4);
    ws.idx = (int *)p;
    p += ((bn * sizeof(int) + 15) / 16) * 16;
    ws.meta = (int2 *)p;
    p += (((size_t)B * T * sizeof(int2) + 15) / 16) * 16;
    ws.rot = (float *)p;
    return ws;
}

hipError_t launch_transform(int B, int N, const float *coords, const float *centers,
                            const float *quats, const float *translations, float *out,
                            hipStream_t stream)
{
    dim3 grid((N + 255) / 256, B);
    hipLaunchKernelGGL(transform_kernel, grid, dim3(256), 0, stream, B, N, coords, centers, quats,
                       translations, out);
    return hipGetLastError();
}

hipError_t launch_prep(const GridSpec &gs, const Batch &bt, const Workspace &ws,
                       float *gclear, float *wclear, hipStream_t stream)
{
    if (bt.weights) {
        hipLaunchKernelGGL(prep_kernel<true>, dim3(1, bt.B), dim3(kPrepThreads), 0, stream, gs, bt,
                           ws, gclear, wclear);
    } else {
        hipLaunchKernelGGL(prep_kernel<false>, dim3(bt.T, bt.B), dim3(kPrepThreads), 0, stream, gs,
                           bt, ws, gclear, wclear);
    }
    return hipGetLastError();
}

}  // namespace mg
