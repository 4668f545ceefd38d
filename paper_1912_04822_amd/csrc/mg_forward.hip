// Steps 3-5 of the path: the forward atom-to-grid kernel (index types, vector
// types, binary occupancy), GridMaker section of the paper.
//
// Design (gfx950, wave64).  The output [B][T][D][D][D] is cut into tiles: a
// tile is `rows` consecutive z-rows of one x-plane of one channel, i.e. one
// contiguous run of rows*D floats (9216 B at D = 48).  A wavefront owns a tile:
//   1. it walks the channel's atom records (written by the prep kernel), 64 at
//      a time, and each lane tests one atom against the tile (disc of the
//      atom's cutoff sphere in this x-plane versus the tile's rows);
//   2. for every atom that passes, the 64 lanes spread over the atom's
//      footprint (rows x 4-voxel z-segments), evaluate the density and add it
//      into the tile held in LDS -- one atom at a time, in record order, so the
//      sum is deterministic and needs no atomics;
//   3. the finished tile is streamed to HBM, each lane writing 32 contiguous
//      bytes (two adjacent 16-byte stores), every output element exactly once,
//      zeros included.  Tiles no atom touches skip LDS and store zeros.
// No barrier is needed: a wavefront only touches its own LDS slice.
//
// The density is rho(x) = exp(-2x^2) for x <= g, A(x-c)^2 for g < x < c, else 0
// (x = d/r); evaluated from x^2 with the hardware exp2 and sqrt.
//
// Binary mode decides d^2 <= r^2 in float with this fixed order (the file is
// compiled with -ffp-contract=off, nothing fuses):
//   gx = o_x + (float)i*res   (o = center - half)      dx = gx - ax
//   d2 = (dx*dx + dy*dy) + dz*dz                        r2 = r*r
#include "mg_common.h"

namespace mg {

namespace {

struct FwdParams {
    GridSpec gs;
    const float4 *rec;
    const int *idx;
    const int2 *meta;
    const float *weights;
    const float *radii;
    const float *centers;
    float *out;
    int B, N, T;
    int rows, strips, pitch;
    long long units;
    int groups;         // workgroups that own tiles
    int xcd_map;
    int debug;
    float kexp;         // -2 * log2(e)
};

__device__ inline float bcast(float v, int src)
{
    return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), src));
}
__device__ inline int bcast(int v, int src) { return __builtin_amdgcn_readlane(v, src); }

// rho as a function of x^2 = d^2 / r^2
__device__ inline float density_from_x2(float x2, float kexp, float g2, float c, float c2, float A)
{
    const float e = __builtin_amdgcn_exp2f(x2 * kexp);
    const float u = __builtin_amdgcn_sqrtf(x2) - c;
    const float q = A * u * u;
    const float v = x2 <= g2 ? e : q;
    return x2 < c2 ? v : 0.0f;
}

template <bool VECTOR, bool BINARY, bool ALIGNED>
__global__ __launch_bounds__(64 * kWavesPerGroup) void forward_kernel(FwdParams p)
{
    __shared__ __attribute__((aligned(16))) float lds[kWavesPerGroup * kTileFloats];

    // grid: x = tile groups of one channel, y = channel, z = example
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const GridSpec &gs = p.gs;
    const int D = gs.D, T = p.T, N = p.N;
    const int uc = (int)blockIdx.x * kWavesPerGroup + wave;     // tile within the channel
    if (uc >= D * p.strips) return;
    const int t = (int)blockIdx.y, b = (int)blockIdx.z;
    const int plane = p.strips == 1 ? uc : uc / p.strips;
    const int strip = p.strips == 1 ? 0 : uc - plane * p.strips;
    float *tile = lds + wave * kTileFloats;
    const int j0 = strip * p.rows;
    const int j1 = min(D, j0 + p.rows);
    const int pitch = p.pitch;

    const float res = gs.res, inv_res = gs.inv_res;
    const float ox = (p.centers ? p.centers[3 * b + 0] : 0.0f) - gs.half;
    const float oy = (p.centers ? p.centers[3 * b + 1] : 0.0f) - gs.half;
    const float oz = (p.centers ? p.centers[3 * b + 2] : 0.0f) - gs.half;
    const float gx = ox + (float)plane * res;

    const int2 m = p.meta[(size_t)b * T + (VECTOR ? 0 : t)];
    const float4 *rec = p.rec + (size_t)b * N + m.x;
    const int *idx = p.idx + (size_t)b * N + m.x;
    const int count = m.y;
    const float r_chan = VECTOR ? gs.radius_scale * p.radii[t] : 0.0f;

    bool any = false;
    for (int base = 0; base < (p.debug == 2 ? 0 : count); base += 64) {
        const int e = base + lane;
        float4 a = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
        float w = 1.0f;
        if (e < count) {
            a = rec[e];
            if (VECTOR && a.w > 0.0f) w = p.weights[((size_t)b * N + idx[e]) * T + t];
        }
        float r = VECTOR ? (a.w > 0.0f ? r_chan : 0.0f) : a.w;
        if (VECTOR) {
            if (BINARY ? !(w > 0.0f) : (w == 0.0f)) r = 0.0f;
        }
        const float reach = BINARY ? r + 1.0e-3f * res : r * gs.c;
        const float dx = gx - a.x;
        const float dx2 = dx * dx;
        const float h2 = reach * reach - dx2;
        bool ok = (r > 0.0f) && (h2 > 0.0f);
        // half-width of the footprint in this plane, in grid steps, padded
        const float hv = __builtin_amdgcn_sqrtf(fmaxf(h2, 0.0f)) * inv_res + 1.0e-3f;
        const float fy = (a.y - oy) * inv_res;
        const float fz = (a.z - oz) * inv_res;
        const int jlo = max(j0, (int)ceilf(fy - hv));
        const int jhi = min(j1 - 1, (int)floorf(fy + hv));
        const int klo = max(0, (int)ceilf(fz - hv));
        const int khi = min(D - 1, (int)floorf(fz + hv));
        ok = ok && (jlo <= jhi) && (klo <= khi);
        const float rr = r * r;
        const float scale = BINARY ? rr : (ok ? 1.0f / rr : 0.0f);   // r^2 or 1/r^2
        const int nrows = jhi - jlo + 1;
        const int seg0 = klo >> 2;
        const int nsegs = (khi >> 2) - seg0 + 1;

        unsigned long long mask = __ballot(ok);
        if (p.debug == 1) mask = 0ull;
        if (mask != 0ull && !any) {
            any = true;
            const float4 z4 = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
            const int n4 = ((j1 - j0) * pitch) >> 2;
            for (int o = lane; o < n4; o += 64) reinterpret_cast<float4 *>(tile)[o] = z4;
            __builtin_amdgcn_wave_barrier();
        }
        while (mask != 0ull) {
            const int src = (int)__builtin_ctzll(mask);
            mask &= mask - 1ull;
            const float ay = bcast(a.y, src), az = bcast(a.z, src);
            const float sdx2 = bcast(dx2, src), sscale = bcast(scale, src);
            const float sw = VECTOR ? bcast(w, src) : 1.0f;
            const int sjlo = bcast(jlo, src), snrows = bcast(nrows, src);
            const int sseg0 = bcast(seg0, src), snsegs = bcast(nsegs, src);
            const int slots = snrows * snsegs;
            const float inv_nsegs = 1.0f / (float)snsegs;
            for (int s = lane; s < slots; s += 64) {
                const int row = (int)(((float)s + 0.5f) * inv_nsegs);
                const int seg = s - row * snsegs;
                const int j = sjlo + row;
                const int k4 = (sseg0 + seg) << 2;
                const float gy = oy + (float)j * res;
                const float dy = gy - ay;
                const float base2 = sdx2 + dy * dy;
                float4 *cell = reinterpret_cast<float4 *>(tile + (j - j0) * pitch + k4);
                float4 v = *cell;
                float vv[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    const float gz = oz + (float)(k4 + u) * res;
                    const float dz = gz - az;
                    const float d2 = base2 + dz * dz;
                    if (BINARY) {
                        if (d2 <= sscale) vv[u] = 1.0f;
                    } else {
                        const float rho = density_from_x2(d2 * sscale, p.kexp, gs.g2, gs.c, gs.c2, gs.A);
                        vv[u] = VECTOR ? fmaf(sw, rho, vv[u]) : vv[u] + rho;
                    }
                }
                *cell = make_float4(vv[0], vv[1], vv[2], vv[3]);
            }
            __builtin_amdgcn_wave_barrier();
        }
    }

    // stream the tile out: every element written exactly once
    float *dst = p.out + ((((size_t)b * T + t) * D + plane) * D + j0) * (size_t)D;
    if (ALIGNED) {
        const int n4 = ((j1 - j0) * D) >> 2;
        float4 *dst4 = reinterpret_cast<float4 *>(dst);
        const float4 *src4 = reinterpret_cast<const float4 *>(tile);
        const float4 z4 = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
        // Constant trip count, fully unrolled, and two separate paths (not a select
        // between an LDS pointer and a zero): a run-time loop bound or a generic-pointer
        // load makes the compiler wait for all earlier stores before each new one.
        constexpr int kIters = (kTileFloats / 4 + 127) / 128;
        if (any) {
            float4 v0[kIters], v1[kIters];
#pragma unroll
            for (int it = 0; it < kIters; ++it) {
                const int o = min(it * 128 + lane * 2, kTileFloats / 4 - 2);
                v0[it] = src4[o];
                v1[it] = src4[o + 1];
            }
#pragma unroll
            for (int it = 0; it < kIters; ++it) {
                const int o = it * 128 + lane * 2;
                if (o < n4) dst4[o] = v0[it];
                if (o + 1 < n4) dst4[o + 1] = v1[it];
            }
        } else {
#pragma unroll
            for (int it = 0; it < kIters; ++it) {
                const int o = it * 128 + lane * 2;
                if (o < n4) dst4[o] = z4;
                if (o + 1 < n4) dst4[o + 1] = z4;
            }
        }
    } else {
        const int n = (j1 - j0) * D;
        for (int o = lane; o < n; o += 64) {
            const int row = o / D;
            const int col = o - row * D;
            dst[o] = any ? tile[row * pitch + col] : 0.0f;
        }
    }
}

}  // namespace

Tiling make_tiling(int B, int T, int D)
{
    Tiling tl;
    tl.pitch = (D + 3) & ~3;
    int rows_max = kTileFloats / tl.pitch;
    if (rows_max < 1) rows_max = 1;
    if (rows_max > D) rows_max = D;
    tl.strips = (D + rows_max - 1) / rows_max;
    tl.rows = (D + tl.strips - 1) / tl.strips;
    tl.units = (long long)B * T * D * tl.strips;
    return tl;
}

hipError_t launch_forward(const GridSpec &gs, const Batch &bt, const Workspace &ws, float *out,
                          int xcd_map, hipStream_t stream)
{
    const Tiling tl = make_tiling(bt.B, bt.T, gs.D);
    FwdParams p;
    p.gs = gs;
    p.rec = ws.rec;
    p.idx = ws.idx;
    p.meta = ws.meta;
    p.weights = bt.weights;
    p.radii = bt.radii;
    p.centers = bt.centers;
    p.out = out;
    p.B = bt.B; p.N = bt.N; p.T = bt.T;
    p.rows = tl.rows; p.strips = tl.strips; p.pitch = tl.pitch;
    p.units = tl.units;
    p.groups = 0;
    p.xcd_map = xcd_map & 1;
    p.debug = xcd_map >> 4;
    p.kexp = -2.8853900817779268f;      // -2 / ln 2
    const int per_channel = (gs.D * tl.strips + kWavesPerGroup - 1) / kWavesPerGroup;
    const bool aligned = (gs.D % 4 == 0) && (((uintptr_t)out & 15u) == 0);
    const bool vec = bt.weights != nullptr;
    const dim3 blk(64 * kWavesPerGroup), grd(per_channel, bt.T, bt.B);
#define MG_LAUNCH(V, Bn, Al) \
    hipLaunchKernelGGL((forward_kernel<V, Bn, Al>), grd, blk, 0, stream, p)
    if (vec) {
        if (gs.binary) { if (aligned) MG_LAUNCH(true, true, true); else MG_LAUNCH(true, true, false); }
        else           { if (aligned) MG_LAUNCH(true, false, true); else MG_LAUNCH(true, false, false); }
    } else {
        if (gs.binary) { if (aligned) MG_LAUNCH(false, true, true); else MG_LAUNCH(false, true, false); }
        else           { if (aligned) MG_LAUNCH(false, false, true); else MG_LAUNCH(false, false, false); }
    }
#undef MG_LAUNCH
    return hipGetLastError();
}

}  // namespace mg
