// Steps 3-5 of the path: the forward atom-to-grid kernel (index types, vector
// types, binary occupancy), GridMaker section of the paper.
//
// Design (gfx950, wave64).  Each channel of the output (D*D*D floats, z fastest)
// is cut into flat tiles of `tile_floats` consecutive floats (2048 = 8192 B by
// default), whatever rows and x-planes that run happens to cover; with the
// usual grids (D = 48, 96) every tile starts on a 4 KB boundary of the output.
// One wavefront produces one tile:
//   1. it loads the records of the channel's atoms that can reach the x-planes
//      the tile touches (spans the prep kernel computed), one atom per lane;
//   2. per x-plane of the tile, each lane tests its atom against the tile's
//      rows in that plane (disc of the atom's cutoff sphere in the plane versus
//      the row range); the (atom, row) pairs that survive are packed into a
//      task list, so that all 64 lanes work even though one atom's footprint is
//      small;
//   3. each lane takes one task: the chord of the atom's sphere along that
//      z-row, clipped to the tile in its first and last row.  It evaluates the
//      density voxel by voxel and adds it into the tile held in LDS with LDS
//      atomics (two atoms may hit one voxel in the same instruction).  The tile
//      accumulates in signed fixed point (2^-24 steps, integer LDS atomics):
//      integer adds run ~40x faster in LDS than float adds on this chip, are
//      exact and order-independent, and a contribution is rounded by at most
//      3e-8.  The sum of the magnitudes that can reach a voxel is tracked; if it
//      could pass 120 (fixed-point range is +-128) the tile switches to float
//      accumulation;
//   4. the finished tile is streamed to HBM, each lane writing 32 contiguous
//      bytes (two adjacent 16-byte stores), every output element exactly once,
//      zeros included.  Tiles no atom touches skip LDS and store zeros.
// No barrier is needed: a wavefront only touches its own LDS slice.
//
// Why 8 KB tiles on 4 KB boundaries: measured on this chip, one-wavefront
// workgroups that each write one aligned 4 KB or 8 KB run sustain 6.3-6.6 TB/s
// at any residency, with or without work between the stores, while runs of
// 6, 9, 18 or 36 KB per wavefront (whole x-planes of a 48^3 grid are 9 KB) fall
// to 5.2-5.4 TB/s.
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

constexpr int kTaskCap = 512;                   // (atom, row) tasks staged per round
constexpr float kFixedOne = 16777216.0f;        // 2^24
constexpr float kFixedLimit = 120.0f;           // largest |sum| trusted to fixed point

struct FwdParams {
    GridSpec gs;
    const float4 *rec;
    const int *idx;
    const int2 *range;
    const float *weights;
    const float *radii;
    const float *centers;
    float *out;
    int B, N, T;
    int tile_floats;    // floats per tile (a multiple of 512)
    int pitch;          // floats per row in LDS
    int tile_lds;       // LDS floats reserved for the tile
    int debug;
    float kexp;         // -2 * log2(e)
};

// what a wavefront keeps for the tile it is working on (all wave-uniform)
struct TileCtx {
    float *tile0;       // LDS: first row of the tile
    int tile_n4;        // float4s of LDS the tile's rows take
    float *tile;        // LDS: row j0 of the current x-plane
    float4 *cand;
    unsigned short *tasks;
    int lane;
    int D, pitch, j0, j1;       // rows [j0, j1) of the current plane belong to the tile
    int jfirst, cfirst;         // row of this plane that is the tile's first row (-1: none) and
    int jlast, clast;           // its first column; same for the last row / last column
    float res, inv_res, oy, oz;
    float g2, c, A, kexp;
    float inv_d4;       // 1 / (D/4)
    int debug;
};

enum TileMode { kUntouched = 0, kFixed = 1, kFloat = 2 };

__device__ inline int bcast(int v, int src) { return __builtin_amdgcn_readlane(v, src); }

// Inclusive prefix sum over the 64 lanes with DPP row shifts and row broadcasts
// (no LDS traffic, six adds).
__device__ inline int wave_inclusive_scan(int v)
{
    v += __builtin_amdgcn_update_dpp(0, v, 0x111, 0xf, 0xf, false);    // row_shr:1
    v += __builtin_amdgcn_update_dpp(0, v, 0x112, 0xf, 0xf, false);    // row_shr:2
    v += __builtin_amdgcn_update_dpp(0, v, 0x114, 0xf, 0xf, false);    // row_shr:4
    v += __builtin_amdgcn_update_dpp(0, v, 0x118, 0xf, 0xf, false);    // row_shr:8
    v += __builtin_amdgcn_update_dpp(0, v, 0x142, 0xa, 0xf, false);    // row_bcast:15 -> rows 1,3
    v += __builtin_amdgcn_update_dpp(0, v, 0x143, 0xc, 0xf, false);    // row_bcast:31 -> rows 2,3
    return v;
}

__device__ inline void lds_sync() { __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront"); }

// rho as a function of x^2 = d^2 / r^2
__device__ inline float density_from_x2(float x2, const TileCtx &cx)
{
    const float e = __builtin_amdgcn_exp2f(x2 * cx.kexp);
    const float u = fminf(__builtin_amdgcn_sqrtf(x2) - cx.c, 0.0f);    // 0 beyond the cutoff
    const float q = cx.A * u * u;
    return x2 <= cx.g2 ? e : q;
}

// Run the staged tasks [0, ntasks): one (atom, row) chord per lane.
template <bool VECTOR, bool BINARY, bool FIXED>
__device__ inline void run_tasks(const TileCtx &cx, int ntasks)
{
    for (int base = 0; base < ntasks; base += 64) {
        const int tau = base + cx.lane;
        bool act = tau < ntasks;
        const int tk = cx.tasks[act ? tau : 0];
        const int cnd = tk & 63, row = tk >> 6;
        const float4 p0 = cx.cand[cnd * 2], p1 = cx.cand[cnd * 2 + 1];
        const float ay = p0.x, az = p0.y, dx2 = p0.z, s = p0.w;
        const float h2 = p1.x, w = p1.y;
        const int j = __float_as_int(p1.z) + row;
        const float gy = cx.oy + (float)j * cx.res;
        const float dy = gy - ay;
        const float dy2 = dy * dy;
        const float rem = h2 - dy2;
        act = act && rem > 0.0f;
        const float hz = __builtin_amdgcn_sqrtf(fmaxf(rem, 0.0f)) * cx.inv_res + 1.0e-3f;
        const float fz = (az - cx.oz) * cx.inv_res;
        // the chord, clipped to the grid and (first / last row of the tile) to the tile
        const int klo = max(j == cx.jfirst ? cx.cfirst : 0, (int)ceilf(fz - hz));
        const int khi = min(j == cx.jlast ? cx.clast : cx.D - 1, (int)floorf(fz + hz));
        const int nz = act ? khi - klo + 1 : 0;
        float *rowp = cx.tile + (j - cx.j0) * cx.pitch + klo;
        if (BINARY) {
            const float base2 = dx2 + dy2;
            for (int i = 0; i < nz; ++i) {
                const float gz = cx.oz + (float)(klo + i) * cx.res;
                const float dz = gz - az;
                const float d2 = base2 + dz * dz;
                if (d2 <= s) rowp[i] = 1.0f;
            }
        } else {
            // coordinates in units of r: x^2 = b2s + zs^2
            const float b2s = (dx2 + dy2) * s * s;
            const float step = cx.res * s;
            const float z0 = ((cx.oz - az) + (float)klo * cx.res) * s;
            for (int i = 0; i < nz; ++i) {
                const float zs = fmaf((float)i, step, z0);
                const float rho = density_from_x2(fmaf(zs, zs, b2s), cx);
                if (FIXED) {
                    const int q = VECTOR ? (int)rintf(w * rho * kFixedOne)
                                         : (int)fmaf(rho, kFixedOne, 0.5f);
                    __hip_atomic_fetch_add(reinterpret_cast<int *>(rowp) + i, q, __ATOMIC_RELAXED,
                                           __HIP_MEMORY_SCOPE_WAVEFRONT);
                } else {
                    __hip_atomic_fetch_add(rowp + i, VECTOR ? w * rho : rho, __ATOMIC_RELAXED,
                                           __HIP_MEMORY_SCOPE_WAVEFRONT);
                }
            }
        }
    }
    lds_sync();
}

// One batch of up to 64 atom records (one per lane) against the rows [j0, j1) of one
// x-plane of the tile.
//   a = {x', y', z', r};  valid: this lane holds a live record;  w: weight (vector types)
//   mode: state of the whole tile;  bound: running bound for this plane
template <bool VECTOR, bool BINARY>
__device__ inline void plane_batch(const TileCtx &cx, float gx, float4 a, float r, float w,
                                   bool valid, int &mode, float &bound)
{
    const float reach = BINARY ? r + 1.0e-3f * cx.res : r * cx.c;
    const float dx = gx - a.x;
    const float dx2 = dx * dx;
    const float h2 = reach * reach - dx2;
    bool ok = valid && (h2 > 0.0f);
    // half-width of the footprint in this plane, in grid steps, padded
    const float hv = __builtin_amdgcn_sqrtf(fmaxf(h2, 0.0f)) * cx.inv_res + 1.0e-3f;
    const float fy = (a.y - cx.oy) * cx.inv_res;
    const float fz = (a.z - cx.oz) * cx.inv_res;
    const int jlo = max(cx.j0, (int)ceilf(fy - hv));
    const int jhi = min(cx.j1 - 1, (int)floorf(fy + hv));
    ok = ok && (jlo <= jhi) && (fz + hv >= 0.0f) && (fz - hv <= (float)(cx.D - 1));
    unsigned long long mask = __ballot(ok);
    if (cx.debug == 1) mask = 0ull;
    if (mask == 0ull) return;

    // upper bound on what this batch can add to one voxel (rho <= 1)
    if (VECTOR) {
        float s = ok ? fabsf(w) : 0.0f;
#pragma unroll
        for (int d = 32; d >= 1; d >>= 1) s += __shfl_xor(s, d, 64);
        bound += s;
    } else {
        bound += (float)__builtin_popcountll(mask);
    }
    if (mode == kUntouched) {
        mode = (BINARY || bound > kFixedLimit) ? kFloat : kFixed;
        const float4 z4 = make_float4(0.0f, 0.0f, 0.0f, 0.0f);     // same bits as integer zeros
        for (int o = cx.lane; o < cx.tile_n4; o += 64) reinterpret_cast<float4 *>(cx.tile0)[o] = z4;
    } else if (mode == kFixed && bound > kFixedLimit) {
        mode = kFloat;                                               // leave fixed point
        for (int o = cx.lane; o < cx.tile_n4 * 4; o += 64)
            cx.tile0[o] = (float)reinterpret_cast<int *>(cx.tile0)[o] * (1.0f / kFixedOne);
    }
    lds_sync();
    const int nrows = ok ? jhi - jlo + 1 : 0;
    if (ok) {
        cx.cand[cx.lane * 2] = make_float4(a.y, a.z, dx2, BINARY ? r * r : 1.0f / r);
        cx.cand[cx.lane * 2 + 1] = make_float4(h2, w, __int_as_float(jlo), 0.0f);
    }
    // exclusive prefix of nrows over the lanes: where each atom's tasks start
    const int incl = wave_inclusive_scan(nrows);
    const int total = bcast(incl, 63);
    if (total <= kTaskCap) {
        const int start = incl - nrows;
        for (int rr = 0; rr < nrows; ++rr) cx.tasks[start + rr] = (unsigned short)(cx.lane | (rr << 6));
        lds_sync();
        if (mode == kFixed) run_tasks<VECTOR, BINARY, true>(cx, total);
        else run_tasks<VECTOR, BINARY, false>(cx, total);
    } else {
        // rare: too many tasks for the staging list; take the atoms one at a time
        while (mask != 0ull) {
            const int src = (int)__builtin_ctzll(mask);
            mask &= mask - 1ull;
            const int n = bcast(nrows, src);
            for (int rr = cx.lane; rr < n; rr += 64) cx.tasks[rr] = (unsigned short)(src | (rr << 6));
            lds_sync();
            if (mode == kFixed) run_tasks<VECTOR, BINARY, true>(cx, n);
            else run_tasks<VECTOR, BINARY, false>(cx, n);
        }
    }
}

// Stream a finished tile to HBM (or zeros if no atom touched it): n floats to dst; the
// first of them sits in column c0 of the tile's first LDS row.
// ITERS = tile_floats / 512: each pass of the wavefront covers 2 KB.
template <bool ALIGNED, int ITERS>
__device__ inline void store_tile(const TileCtx &cx, float *dst, int c0, int n, int mode)
{
    if (ALIGNED) {
        const int n4 = n >> 2;                      // even: D^3 and the tile size are multiples of 8
        const int d4 = cx.D >> 2, p4 = cx.pitch >> 2, q0 = c0 >> 2;
        float4 *dst4 = reinterpret_cast<float4 *>(dst);
        const float4 *src4 = reinterpret_cast<const float4 *>(cx.tile0);
        const float4 z4 = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
        // Constant trip count, fully unrolled; the tile comes from LDS into registers
        // under a wave-uniform branch (zeros otherwise), so that the stores below are one
        // straight sequence with no load between them.
        float4 v[2 * ITERS];
        if (mode != kUntouched) {
#pragma unroll
            for (int it = 0; it < 2 * ITERS; ++it) {
                const int o = min((it >> 1) * 128 + cx.lane * 2 + (it & 1), n4 - 1) + q0;
                const int row = (int)(((float)o + 0.5f) * cx.inv_d4);
                v[it] = src4[row * p4 + (o - row * d4)];            // rows are padded in LDS
            }
            if (mode == kFixed) {
#pragma unroll
                for (int it = 0; it < 2 * ITERS; ++it) {
                    const float sc = 1.0f / kFixedOne;
                    v[it] = make_float4((float)__float_as_int(v[it].x) * sc,
                                        (float)__float_as_int(v[it].y) * sc,
                                        (float)__float_as_int(v[it].z) * sc,
                                        (float)__float_as_int(v[it].w) * sc);
                }
            }
        } else {
#pragma unroll
            for (int it = 0; it < 2 * ITERS; ++it) v[it] = z4;
        }
        // the two 16-byte halves of a lane's 32 bytes go out back to back, under one
        // predicate: separated by other instructions they are markedly slower
#pragma unroll
        for (int it = 0; it < ITERS; ++it) {
            const int o = it * 128 + cx.lane * 2;
            if (o < n4) {
                dst4[o] = v[2 * it];
                dst4[o + 1] = v[2 * it + 1];
            }
        }
    } else {
        for (int o = cx.lane; o < n; o += 64) {
            const int f = o + c0;
            const int row = f / cx.D;
            const int col = f - row * cx.D;
            float v = 0.0f;
            if (mode == kFloat) v = cx.tile0[row * cx.pitch + col];
            if (mode == kFixed)
                v = (float)reinterpret_cast<const int *>(cx.tile0)[row * cx.pitch + col] *
                    (1.0f / kFixedOne);
            dst[o] = v;
        }
    }
}

template <bool VECTOR, bool BINARY, bool ALIGNED, int ITERS>
__global__ __launch_bounds__(64) void forward_kernel(FwdParams p)
{
    extern __shared__ __attribute__((aligned(16))) float lds[];   // tile | candidates | tasks

    // grid: x = tile of one channel, y = channel, z = example; one wavefront each
    const int lane = threadIdx.x;
    const GridSpec &gs = p.gs;
    const int D = gs.D, T = p.T, N = p.N;
    const int t = (int)blockIdx.y, b = (int)blockIdx.z;

    // the tile: floats [f0, f1) of the channel = rows [R0, R1) of its D*D rows, the first
    // from column c0 on, the last up to column c1
    const int total = D * D * D;
    const int f0 = (int)blockIdx.x * p.tile_floats;
    const int f1 = min(total, f0 + p.tile_floats);
    const int R0 = f0 / D, R1 = (f1 - 1) / D + 1;
    const int c0 = f0 - R0 * D, c1 = f1 - 1 - (R1 - 1) * D;
    const int i_lo = R0 / D, i_hi = (R1 - 1) / D;

    TileCtx cx;
    cx.tile0 = lds;
    cx.tile_n4 = ((R1 - R0) * p.pitch) >> 2;
    cx.tile = lds;
    cx.cand = reinterpret_cast<float4 *>(lds + p.tile_lds);
    cx.tasks = reinterpret_cast<unsigned short *>(lds + p.tile_lds + 64 * 8);
    cx.lane = lane;
    cx.D = D;
    cx.pitch = p.pitch;
    cx.j0 = 0;
    cx.j1 = 0;
    cx.jfirst = -1; cx.cfirst = c0;
    cx.jlast = -1; cx.clast = c1;
    cx.res = gs.res;
    cx.inv_res = gs.inv_res;
    cx.g2 = gs.g2; cx.c = gs.c; cx.A = gs.A; cx.kexp = p.kexp;
    cx.inv_d4 = 1.0f / (float)max(1, D >> 2);
    cx.debug = p.debug;

    float *dst = p.out + ((size_t)b * T + t) * (size_t)total + f0;
    if (p.debug == 3) {         // timing aid: nothing but the zero stores
        store_tile<ALIGNED, ITERS>(cx, dst, c0, f1 - f0, kUntouched);
        return;
    }
    const size_t group = (size_t)b * T + (VECTOR ? 0 : t);
    // records (relative to the example's first) that can reach planes i_lo .. i_hi
    const int r0 = p.range[group * D + i_lo].x;
    const int r1 = p.debug == 2 ? r0 : p.range[group * D + i_hi].y;
    const float ox = (p.centers ? p.centers[3 * b + 0] : 0.0f) - gs.half;
    cx.oy = (p.centers ? p.centers[3 * b + 1] : 0.0f) - gs.half;
    cx.oz = (p.centers ? p.centers[3 * b + 2] : 0.0f) - gs.half;
    const float r_chan = VECTOR ? gs.radius_scale * p.radii[t] : 0.0f;

    const float4 *rec = p.rec + (size_t)b * N + r0;
    const int *idx = p.idx + (size_t)b * N + r0;
    const int count = r1 - r0;

    // the usual case: every atom that can reach the tile sits in one lane, loaded once
    const bool once = count <= 64;
    float4 a = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
    float w = 1.0f;
    if (once && lane < count) {
        a = rec[lane];
        if (VECTOR && a.w > 0.0f) w = p.weights[((size_t)b * N + idx[lane]) * T + t];
    }
    float r = VECTOR ? r_chan : a.w;
    bool valid = (lane < count) && (a.w > 0.0f) && (r > 0.0f);
    if (VECTOR) valid = valid && (BINARY ? (w > 0.0f) : (w != 0.0f));

    int mode = kUntouched;
    for (int i = i_lo; i <= i_hi && count > 0; ++i) {
        // rows of plane i inside the tile
        const int ja = max(R0 - i * D, 0), jb = min(R1 - i * D, D);
        cx.j0 = ja;
        cx.j1 = jb;
        cx.tile = cx.tile0 + (i * D + ja - R0) * p.pitch;
        cx.jfirst = (i == i_lo) ? ja : -1;
        cx.jlast = (i == i_hi) ? jb - 1 : -1;
        const float gx = ox + (float)i * gs.res;
        float bound = 0.0f;         // planes do not share voxels: one bound per plane
        if (once) {
            plane_batch<VECTOR, BINARY>(cx, gx, a, r, w, valid, mode, bound);
        } else {
            for (int base = 0; base < count; base += 64) {
                const int e = base + lane;
                a = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
                w = 1.0f;
                if (e < count) {
                    a = rec[e];
                    if (VECTOR && a.w > 0.0f) w = p.weights[((size_t)b * N + idx[e]) * T + t];
                }
                r = VECTOR ? r_chan : a.w;
                valid = (e < count) && (a.w > 0.0f) && (r > 0.0f);
                if (VECTOR) valid = valid && (BINARY ? (w > 0.0f) : (w != 0.0f));
                plane_batch<VECTOR, BINARY>(cx, gx, a, r, w, valid, mode, bound);
            }
        }
    }
    store_tile<ALIGNED, ITERS>(cx, dst, c0, f1 - f0, mode);
}

}  // namespace

ForwardGeometry forward_geometry(int D, int tile_floats)
{
    ForwardGeometry fg;
    fg.tile_floats = tile_floats;
    const long long total = (long long)D * D * D;
    fg.tiles = (int)((total + tile_floats - 1) / tile_floats);
    // LDS rows are padded by 4 floats: with a pitch of D (a multiple of 16 for the usual
    // grids) the rows of one atom would fall on a few LDS banks only
    fg.pitch = ((D + 3) & ~3) + 4;
    // a run of tile_floats floats touches at most tile_floats/D + 2 rows
    long long rows = (long long)tile_floats / D + 2;
    if (rows > (long long)D * D) rows = (long long)D * D;
    fg.tile_lds = (int)((rows * fg.pitch + 3) & ~3LL);
    return fg;
}

hipError_t launch_forward(const GridSpec &gs, const Batch &bt, const Workspace &ws, float *out,
                          int tile_floats, int lds_pad, int debug, hipStream_t stream)
{
    const ForwardGeometry fg = forward_geometry(gs.D, tile_floats);
    FwdParams p;
    p.gs = gs;
    p.rec = ws.rec;
    p.idx = ws.idx;
    p.range = ws.range;
    p.weights = bt.weights;
    p.radii = bt.radii;
    p.centers = bt.centers;
    p.out = out;
    p.B = bt.B; p.N = bt.N; p.T = bt.T;
    p.tile_floats = fg.tile_floats;
    p.pitch = fg.pitch;
    p.tile_lds = fg.tile_lds;
    p.debug = debug;
    p.kexp = -2.8853900817779268f;      // -2 / ln 2
    const size_t lds_bytes = ((size_t)p.tile_lds + 64 * 8 + kTaskCap / 2) * sizeof(float) + lds_pad;
    const bool aligned = (gs.D % 4 == 0) && (((uintptr_t)out & 15u) == 0);
    const bool vec = bt.weights != nullptr;
    const dim3 blk(64), grd(fg.tiles, bt.T, bt.B);
#define MG_LAUNCH4(V, Bn, Al, It) \
    hipLaunchKernelGGL((forward_kernel<V, Bn, Al, It>), grd, blk, lds_bytes, stream, p)
#define MG_LAUNCH(V, Bn, Al)                            \
    switch (tile_floats) {                              \
    case 512: MG_LAUNCH4(V, Bn, Al, 1); break;          \
    case 1024: MG_LAUNCH4(V, Bn, Al, 2); break;         \
    case 2048: MG_LAUNCH4(V, Bn, Al, 4); break;         \
    case 4096: MG_LAUNCH4(V, Bn, Al, 8); break;         \
    default: return hipErrorInvalidValue;               \
    }
    if (vec) {
        if (gs.binary) { if (aligned) MG_LAUNCH(true, true, true) else MG_LAUNCH(true, true, false) }
        else           { if (aligned) MG_LAUNCH(true, false, true) else MG_LAUNCH(true, false, false) }
    } else {
        if (gs.binary) { if (aligned) MG_LAUNCH(false, true, true) else MG_LAUNCH(false, true, false) }
        else           { if (aligned) MG_LAUNCH(false, false, true) else MG_LAUNCH(false, false, false) }
    }
#undef MG_LAUNCH
#undef MG_LAUNCH4
    return hipGetLastError();
}

}  // namespace mg
