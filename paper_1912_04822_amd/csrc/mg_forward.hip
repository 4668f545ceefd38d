// Steps 3-5 of the path: the forward atom-to-grid kernel (index types, vector
// types, binary occupancy), GridMaker section of the paper.
//
// Design (gfx950, wave64).  Each channel of the output (D*D*D floats, z fastest)
// is cut into flat tiles of `tile_floats` consecutive floats (1024 = 4096 B by
// default, 2048 when a tile is expected to meet many records), whatever rows and
// x-planes that run happens to cover; with the usual grids (D = 48, 96) every
// tile starts on a 4 KB boundary of the output.
// One workgroup of 1, 2 or 4 wavefronts produces one tile; its wavefronts split
// the atoms and, at the end, the 2 KB chunks of the tile between them:
//   1. the workgroup loads the records of the channel's atoms that can reach the
//      x-planes the tile touches (spans the prep kernel computed), one atom per
//      lane, atom e going to wavefront e mod (number of wavefronts);
//   2. each lane tests its atom against the tile's rows in two x-planes at a
//      time (disc of the atom's cutoff sphere in the plane versus the row
//      range).  Every surviving (atom, row) pair is a task; a wavefront scan
//      gives each atom the index of its first task, which the lane marks in a
//      byte array, so that a later max-scan over the marks tells every lane
//      which atom its task belongs to: all 64 lanes work even though one
//      atom's footprint is small, and no lane loops over its rows to list them;
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
// The tile sits in LDS in output order (LDS index = output index - first index of
// the tile).  With more than one wavefront there are two barriers per tile: after
// the zero fill and the decision between fixed point and float (which needs the
// bound over all wavefronts), and before the tile is read back.  The default is
// one wavefront per 4 KB tile (no barrier at all; 8 KB when a tile meets many
// records).  A grid of doubles takes 512 voxels per workgroup (4 KB of output) and
// stores 1 KB per instruction.
//
// Why 4 KB / 8 KB tiles on 4 KB boundaries: measured on this chip, one-wavefront
// workgroups that each write one aligned 4 KB or 8 KB run sustain 6.3-6.6 TB/s
// when nothing else is going on, while runs of 6, 9, 18 or 36 KB per wavefront
// (whole x-planes of a 48^3 grid are 9 KB) fall to 5.2-5.4 TB/s.  Reads do not
// disturb that stream as long as a cache serves them; reads that must come from
// HBM do, far beyond their bytes.  The tables this kernel reads (a few MB, written
// by the prep kernel just before) would be pushed out to HBM by the hundreds of MB
// of stores before the later examples' turn, so every wavefront also touches 1 KB
// of them (see the kernel's preamble): 102 us against 108 us per launch on the
// 48^3 batch of 50, 257 us against 328 us on a 96^3 batch of 16.
//
// The density is rho(x) = exp(-2x^2) for x <= g, A(x-c)^2 for g < x < c, else 0
// (x = d/r).  Distances are carried in units of r/sqrt(k), k = 2*log2(e), so
// that the Gaussian is exp2(-x'^2) with the hardware exp2 and the tail is
// (sqrt(x'^2)*sA - cA)^2 with sA = sqrt(A/k), cA = c*sqrt(A).
//
// Binary mode decides d^2 <= r^2 in float with this fixed order (the file is
// compiled with -ffp-contract=off, nothing fuses):
//   gx = o_x + (float)i*res   (o = center - half)      dx = gx - ax
//   d2 = (dx*dx + dy*dy) + dz*dz                        r2 = r*r
#include <cmath>

#include "mg_common.h"
#include "mg_wave.h"
#include "mg_xform.h"

namespace mg {

namespace {

constexpr int kTaskCap = 256;                   // (atom, row) tasks staged per round
constexpr unsigned kKeepAliveBytes = 256;       // what every wavefront re-reads of the tables by default
constexpr float kFixedOne = 16777216.0f;        // 2^24
constexpr float kFixedLimit = 120.0f;           // largest |sum| trusted to fixed point

// The caller's arrays, for the single-launch path of small problems (no prep kernel, no tables).
struct RawInputs {
    const float *coords;
    const int32_t *types;
    const float *radii;
    const int32_t *natoms;
    const float *centers, *quats, *translations;
};

struct FwdParams {
    GridSpec gs;
    RawInputs raw;
    const float4 *rec;
    const int *idx;
    const int2 *range;
    const float *weights;
    const float *radii;
    const float *gcen;          // [B][4] grid centres, written by the prep kernel
    const int *chan_order;      // [B][T] vector types: channels in order of radius
    unsigned groups;            // vector types: groups of kVecGroup channels per example
    const unsigned *tag;        // what the workspace's tables were made for
    unsigned expect_tag;        // != 0: do nothing unless *tag equals it (calls on prepared tables)
    void *out;                      // float or double grid
    int subgrids, N, T;             // subgrids: virtual examples per example (weights are per example)
    int tile_floats;                // floats per tile (a multiple of 512)
    unsigned tiles;                 // divisor of the workgroup id: tiles per channel, or channels (B*T) when pos_major
    unsigned pos_major;             // 0: all tiles of a channel, then the next channel; 1: tile k of every channel, then tile k+1
    unsigned long long div_magic;   // ceil(2^40 / D): x / D = (x * div_magic) >> 40 for x < D^3
    unsigned long long tiles_magic; // ceil(2^64 / tiles), see div_u32
    unsigned long long t_magic;     // ceil(2^64 / T)
    int xcd_shift;                  // >= 0: runs of 2^xcd_shift consecutive tiles go to one XCD
    unsigned n_remap;               // workgroups covered by that mapping (the rest map 1:1)
    int debug;
    unsigned ka_chunks, ka_last;    // keep-alive reads: chunks of the tables (0: none), byte offset of the last one
    unsigned ka_shift;              // log2 of the chunk size in bytes (6..10)
    unsigned ka_skip;               // 0, 1, 3 or 7: wavefronts whose id has none of these bits set do the read
    float sk;           // sqrt(k), k = 2 log2(e)
    float inv_sk;
    float g2k, c2k;     // g^2 k, c^2 k
    float sA, cA;       // tail coefficients
};

// what a wavefront keeps for the tile it is working on (all wave-uniform)
struct TileCtx {
    float *tile;                // LDS: tile_floats floats, in output order
    unsigned char *marks;       // LDS (per wavefront): marks[first task of the atom in lane l] = l + 1
    int *shared;                // LDS (workgroup): [0] bound on |sum| (1/256 units), [1] any task
    int lane, wave;
    int D, n;                   // points per side; floats in this tile
    int nrows;                  // grid rows the tile touches
    int c0, c1;                 // first column of its first row, last column of its last row
    int rowA, rowB;             // tile row of row 0 of plane A / plane B (may be negative)
    float res, inv_res, oy, oz;     // oy, oz: grid origin (binary mode works from it)
    float cen_x, cen_y, cen_z, hD;  // grid centre; (D-1)/2.  The real density works in
                                    // coordinates relative to the centre: differences of
                                    // nearby numbers, no rounding of an origin
    float g2k, c2k, sA, cA;
    int debug;
};

enum TileMode { kUntouched = 0, kFixed = 1, kFloat = 2 };

__device__ inline int div_by_d(int x, unsigned long long magic)
{
    return (int)(((unsigned long long)(unsigned)x * magic) >> 40);
}

// x / d for any 32-bit x, with magic = ceil(2^64 / d) (d >= 2; d == 1 is passed as magic 0).
__device__ inline unsigned div_u32(unsigned x, unsigned long long magic)
{
    return magic == 0ull ? x : (unsigned)__umul64hi((unsigned long long)x, magic);
}

// One atom of the current batch as its lane holds it.
struct Atom {
    float4 a;           // x', y', z', r
    float w;            // weight (vector types), else 1
    bool valid;
};

// What a task needs of its atom; it stays in the registers of the atom's lane and the
// task's lane fetches it with ds_bpermute (register exchange, no LDS storage).
struct Cand {
    float c0, c1, c2, c3;       // fy, fz (grid steps from the centre), stepk, inv_stepk | w
                                // (binary: y', z', r^2, reach^2)
    float pxA, pxB;             // plane term of d^2 for plane A, plane B
    int start;                  // index of the atom's first task
    int pack;                   // jloA | nA << 10 | jloB << 20
};

__device__ inline float fetch(int byte_addr, float v)
{
    return __int_as_float(__builtin_amdgcn_ds_bpermute(byte_addr, __float_as_int(v)));
}

// Run the staged tasks [0, ntasks): one (atom, row) chord per lane.
template <bool BINARY, bool FIXED>
__device__ inline void run_tasks(const TileCtx &cx, const Cand &cd, int ntasks)
{
    int carry = 0;
    for (int base = 0; base < ntasks; base += 64) {
        const int tau = base + cx.lane;
        bool act = tau < ntasks;
        // which atom: the last mark at or before this task
        const int owner = max(carry, wave_inclusive_max((int)cx.marks[tau]));
        carry = bcast(owner, 63);
        const int src = (act ? owner - 1 : 0) << 2;
        const float4 p0 = make_float4(fetch(src, cd.c0), fetch(src, cd.c1), fetch(src, cd.c2),
                                      fetch(src, cd.c3));
        const float2 p1 = make_float2(fetch(src, cd.pxA), fetch(src, cd.pxB));
        const int pack = __builtin_amdgcn_ds_bpermute(src, cd.pack);
        const int k = tau - __builtin_amdgcn_ds_bpermute(src, cd.start);   // row number within the atom
        const int nA = (pack >> 10) & 1023;
        const bool inB = k >= nA;
        const int j = inB ? (pack >> 20) + (k - nA) : (pack & 1023) + k;   // row in its plane
        const int trow = (inB ? cx.rowB : cx.rowA) + j;                    // row in the tile
        const float px2 = inB ? p1.y : p1.x;                               // plane term of d^2
        const int clip_lo = trow == 0 ? cx.c0 : 0;
        const int clip_hi = trow == cx.nrows - 1 ? cx.c1 : cx.D - 1;
        float *rowp = cx.tile + (trow * cx.D - cx.c0);
        if (BINARY) {
            const float ay = p0.x, az = p0.y, r2 = p0.z, reach2 = p0.w;
            const float gy = cx.oy + (float)j * cx.res;
            const float dy = gy - ay;
            const float dy2 = dy * dy;
            const float rem = (reach2 - px2) - dy2;
            act = act && rem > 0.0f;
            const float hz = __builtin_amdgcn_sqrtf(fmaxf(rem, 0.0f)) * cx.inv_res + 1.0e-3f;
            const float fz = (az - cx.oz) * cx.inv_res;
            const int klo = max(clip_lo, (int)ceilf(fz - hz));
            const int khi = min(clip_hi, (int)floorf(fz + hz));
            const int nz = act ? khi - klo + 1 : 0;
            const float base2 = px2 + dy2;
            for (int i = 0; i < nz; ++i) {
                const float gz = cx.oz + (float)(klo + i) * cx.res;
                const float dz = gz - az;
                const float d2 = base2 + dz * dz;
                if (d2 <= r2) rowp[klo + i] = 1.0f;
            }
        } else {
            const float fy = p0.x, fz = p0.y, stepk = p0.z, inv_stepk = p0.w;
            const float dyk = (((float)j - cx.hD) - fy) * stepk;
            const float x2b = fmaf(dyk, dyk, px2);
            const float rem = cx.c2k - x2b;
            act = act && rem > 0.0f;
            const float hz = __builtin_amdgcn_sqrtf(fmaxf(rem, 0.0f)) * inv_stepk + 1.0e-3f;
            const float fzi = fz + cx.hD;                                   // as a grid index
            const int klo = max(clip_lo, (int)ceilf(fzi - hz));
            const int khi = min(clip_hi, (int)floorf(fzi + hz));
            const int nz = act ? khi - klo + 1 : 0;
            const float z0 = (((float)klo - cx.hD) - fz) * stepk;
            float cA = cx.cA;
            asm volatile("" : "+v"(cA));        // keep it in a VGPR across the loop
            float fi = 0.0f;
            for (int i = 0; i < nz; ++i) {
                const float zs = fmaf(fi, stepk, z0);
                fi += 1.0f;
                const float x2 = fmaf(zs, zs, x2b);
                const float e = __builtin_amdgcn_exp2f(-x2);
                // sqrt(A) (c - x), at most exp(-g^2) <= 1 where the tail applies: the multiply-add's
                // clamp to [0, 1] cuts it off at the cutoff
                const float u = __builtin_amdgcn_fmed3f(fmaf(-__builtin_amdgcn_sqrtf(x2), cx.sA, cA), 0.0f, 1.0f);
                const float rho = x2 <= cx.g2k ? e : u * u;             // 0 beyond the cutoff
                if (FIXED) {
                    __hip_atomic_fetch_add(reinterpret_cast<int *>(rowp) + klo + i,
                                           (int)fmaf(rho, kFixedOne, 0.5f), __ATOMIC_RELAXED,
                                           __HIP_MEMORY_SCOPE_WORKGROUP);
                } else {
                    __hip_atomic_fetch_add(rowp + klo + i, rho, __ATOMIC_RELAXED,
                                           __HIP_MEMORY_SCOPE_WORKGROUP);
                }
            }
        }
    }
    lds_sync();
}

// Rows of one x-plane (rows [ja, jb) of it belong to the tile) that the lane's atom reaches.
//   out: px2 = plane term of the squared distance (scaled units; binary: dx^2), rows [jlo, jlo+n)
template <bool BINARY>
__device__ inline int plane_rows(const TileCtx &cx, const FwdParams &p, const Atom &at, float gx,
                                 float xc, int ja, int jb, float sks, float inv_stepk, float fy,
                                 float fz, float &px2, int &jlo)
{
    // gx: x of the plane; xc: the same relative to the grid centre; fy, fz: grid indices
    float hv;
    bool ok = at.valid && ja < jb;
    if (BINARY) {
        const float dx = gx - at.a.x;
        const float reach = at.a.w + 1.0e-3f * cx.res;
        px2 = dx * dx;
        const float h2 = reach * reach - px2;
        ok = ok && h2 > 0.0f;
        hv = __builtin_amdgcn_sqrtf(fmaxf(h2, 0.0f)) * cx.inv_res + 1.0e-3f;
    } else {
        const float dxk = (xc - (at.a.x - cx.cen_x)) * sks;
        px2 = dxk * dxk;
        const float h2 = cx.c2k - px2;
        ok = ok && h2 > 0.0f;
        hv = __builtin_amdgcn_sqrtf(fmaxf(h2, 0.0f)) * inv_stepk + 1.0e-3f;
    }
    // half-width of the footprint in this plane, in grid steps, padded
    jlo = max(ja, (int)ceilf(fy - hv));
    const int jhi = min(jb - 1, (int)floorf(fy + hv));
    ok = ok && (jlo <= jhi) && (fz + hv >= 0.0f) && (fz - hv <= (float)(cx.D - 1));
    return ok ? jhi - jlo + 1 : 0;
}

// What one lane found for its atom in planes iA and iA + 1 of the tile.
struct PairHit {
    Cand cd;
    int nA, nB;         // rows reached in plane A, plane B
};

// One atom per lane against the rows of planes A and B that belong to the tile.
template <bool BINARY>
__device__ inline PairHit pair_test(const TileCtx &cx, const FwdParams &p, const Atom &at, float ox,
                                    int iA, int jaA, int jbA, int jaB, int jbB)
{
    PairHit h;
    const float r = at.a.w;
    // per atom: position in grid steps, scale of its distances
    const float fy = (at.a.y - cx.cen_y) * cx.inv_res;      // from the grid centre
    const float fz = (at.a.z - cx.cen_z) * cx.inv_res;
    const float fyi = BINARY ? (at.a.y - cx.oy) * cx.inv_res : fy + cx.hD;   // as grid indices
    const float fzi = BINARY ? (at.a.z - cx.oz) * cx.inv_res : fz + cx.hD;
    const float sks = at.valid ? p.sk * __builtin_amdgcn_rcpf(r) : 0.0f;
    const float stepk = cx.res * sks;
    const float inv_stepk = r * cx.inv_res * p.inv_sk;
    int jloA, jloB = 0;
    const float gxA = ox + (float)iA * cx.res, gxB = ox + (float)(iA + 1) * cx.res;
    const float xcA = ((float)iA - cx.hD) * cx.res, xcB = ((float)(iA + 1) - cx.hD) * cx.res;
    h.nA = plane_rows<BINARY>(cx, p, at, gxA, xcA, jaA, jbA, sks, inv_stepk, fyi, fzi, h.cd.pxA, jloA);
    h.nB = 0;
    h.cd.pxB = 0.0f;
    if (jaB < jbB)      // uniform: most tiles of small tile sizes lie in one plane
        h.nB = plane_rows<BINARY>(cx, p, at, gxB, xcB, jaB, jbB, sks, inv_stepk, fyi, fzi, h.cd.pxB, jloB);
    if (MG_DEBUG_IS(cx, 1)) { h.nA = 0; h.nB = 0; }
    if (h.nA == 0) jloA = 0;        // both are packed into bit fields below
    if (h.nB == 0) jloB = 0;
    if (BINARY) {
        const float reach = r + 1.0e-3f * cx.res;
        h.cd.c0 = at.a.y; h.cd.c1 = at.a.z; h.cd.c2 = r * r; h.cd.c3 = reach * reach;
    } else {
        h.cd.c0 = fy; h.cd.c1 = fz; h.cd.c2 = stepk; h.cd.c3 = inv_stepk;
    }
    h.cd.start = 0;
    h.cd.pack = jloA | (h.nA << 10) | (jloB << 20);
    return h;
}

// What the hits of this wavefront can add to one voxel at most (rho <= 1), in 1/256.
template <bool VECTOR>
__device__ inline int pair_bound(const PairHit &h, const Atom &at)
{
    const bool hit = h.nA + h.nB > 0;
    if (VECTOR) {       // each weight rounded up to 1/256, summed exactly by DPP adds (no LDS traffic)
        const int mine = hit ? (int)ceilf(fminf(fabsf(at.w), 4096.0f) * 256.0f) : 0;
        return bcast(wave_inclusive_scan(mine), 63);
    }
    return 256 * (int)__builtin_popcountll(__ballot(hit));
}

// Stage the tasks of the hits (rows of plane A, then rows of plane B, atom after atom)
// and run them.
// Returns whether there was any task.
template <bool BINARY>
__device__ inline bool pair_run(const TileCtx &cx, PairHit &h, bool fixed)
{
    int todo = h.nA + h.nB;         // lanes still to be staged have todo > 0
    if (__ballot(todo > 0) == 0ull) return false;
    while (true) {
        const int incl = wave_inclusive_scan(todo);
        int total = bcast(incl, 63);
        if (total == 0) break;
        bool now = todo > 0;
        if (total > kTaskCap) {     // rare: the rest waits for the next round
            now = now && incl <= kTaskCap;
            total = bcast(wave_inclusive_scan(now ? todo : 0), 63);
            if (total == 0) break;
        }
        if (cx.lane < kTaskCap / 16)
            reinterpret_cast<float4 *>(cx.marks)[cx.lane] = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
        if (now) {
            h.cd.start = incl - todo;
            cx.marks[h.cd.start] = (unsigned char)(cx.lane + 1);
            todo = 0;
        }
        lds_sync();
        if (fixed) run_tasks<BINARY, true>(cx, h.cd, total);
        else run_tasks<BINARY, false>(cx, h.cd, total);
    }
    return true;
}

// Stream the finished tile to HBM (zeros if no atom touched it).  ITERS = tile_floats / 512
// chunks of 2 KB; wavefront w of NW takes chunks w, w + NW, ...
template <bool ALIGNED, int ITERS, int NW, typename OUT>
__device__ inline void store_tile(const TileCtx &cx, OUT *dst, bool touched, bool fixed)
{
    constexpr bool kWide = sizeof(OUT) == 8;        // a grid of doubles: the same values, widened
    if (ALIGNED && kWide) {
        // Doubles: every store instruction writes 1 KB in one piece (lane l its 16 bytes at
        // 16 l), four per 512-voxel chunk.
        constexpr int MINE = ITERS / NW;
        const int n2 = cx.n >> 1;
        double2 *dst2 = reinterpret_cast<double2 *>(dst);
        const float2 *src2 = reinterpret_cast<const float2 *>(cx.tile);
        const bool convert = touched && fixed;
#pragma unroll
        for (int it = 0; it < MINE; ++it) {
            float2 v[4];
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                const int o = ((it * NW + cx.wave) * 4 + k) * 64 + cx.lane;
                v[k] = touched ? src2[o] : make_float2(0.0f, 0.0f);
                if (convert) {
                    const float sc = 1.0f / kFixedOne;
                    v[k] = make_float2((float)__float_as_int(v[k].x) * sc,
                                       (float)__float_as_int(v[k].y) * sc);
                }
            }
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                const int o = ((it * NW + cx.wave) * 4 + k) * 64 + cx.lane;
                if (o < n2) dst2[o] = make_double2((double)v[k].x, (double)v[k].y);
            }
        }
    } else if (ALIGNED) {
        constexpr int MINE = ITERS / NW;            // chunks per wavefront
        const int n4 = cx.n >> 2;                   // even: D^3 and the tile size are multiples of 8
        float4 *dst4 = reinterpret_cast<float4 *>(dst);         // float grids
        double2 *dst2 = reinterpret_cast<double2 *>(dst);       // double grids
        const float4 *src4 = reinterpret_cast<const float4 *>(cx.tile);
        // Constant trip count, fully unrolled; the tile comes from LDS into registers
        // under a uniform branch (zeros otherwise), so that the stores below are one
        // straight sequence with no load between them.
        float4 v[2 * MINE];
        if (touched) {
#pragma unroll
            for (int it = 0; it < 2 * MINE; ++it)
                v[it] = src4[((it >> 1) * NW + cx.wave) * 128 + cx.lane * 2 + (it & 1)];
        } else {
#pragma unroll
            for (int it = 0; it < 2 * MINE; ++it) v[it] = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
        }
        const bool convert = touched && fixed;
        // chunk after chunk: convert its two float4s, then the two 16-byte halves of a lane's
        // 32 bytes go out back to back, under one predicate (separated by other instructions
        // they are markedly slower); the first stores leave while later chunks are converted
#pragma unroll
        for (int it = 0; it < MINE; ++it) {
            float4 a = v[2 * it], b = v[2 * it + 1];
            if (convert) {
                const float sc = 1.0f / kFixedOne;
                a = make_float4((float)__float_as_int(a.x) * sc, (float)__float_as_int(a.y) * sc,
                                (float)__float_as_int(a.z) * sc, (float)__float_as_int(a.w) * sc);
                b = make_float4((float)__float_as_int(b.x) * sc, (float)__float_as_int(b.y) * sc,
                                (float)__float_as_int(b.z) * sc, (float)__float_as_int(b.w) * sc);
            }
            const int o = (it * NW + cx.wave) * 128 + cx.lane * 2;
            if (o < n4) {
                if (kWide) {        // the lane's 8 values are 64 contiguous bytes: four 16-byte stores
                    dst2[2 * o] = make_double2((double)a.x, (double)a.y);
                    dst2[2 * o + 1] = make_double2((double)a.z, (double)a.w);
                    dst2[2 * o + 2] = make_double2((double)b.x, (double)b.y);
                    dst2[2 * o + 3] = make_double2((double)b.z, (double)b.w);
                } else {
                    dst4[o] = a;
                    dst4[o + 1] = b;
                }
            }
        }
    } else {
        for (int o = cx.wave * 64 + cx.lane; o < cx.n; o += 64 * NW) {
            float v = 0.0f;
            if (touched)
                v = fixed ? (float)reinterpret_cast<const int *>(cx.tile)[o] * (1.0f / kFixedOne)
                          : cx.tile[o];
            dst[o] = (OUT)v;
        }
    }
}

// Where a tile lies: floats [f0, f1) of the channel = rows [R0, R1) of its D*D rows, which
// belong to x-planes i_lo .. i_hi.
struct TileGeom {
    int f0, f1, R0, R1, i_lo, i_hi;
};

template <int ITERS>
__device__ inline TileGeom tile_geom(const FwdParams &p, int D, unsigned tile_in_chan)
{
    TileGeom g;
    const int total = D * D * D;
    g.f0 = (int)tile_in_chan * (ITERS * 512);
    g.f1 = min(total, g.f0 + ITERS * 512);
    g.R0 = div_by_d(g.f0, p.div_magic);
    g.R1 = div_by_d(g.f1 - 1, p.div_magic) + 1;
    g.i_lo = div_by_d(g.R0, p.div_magic);
    g.i_hi = div_by_d(g.R1 - 1, p.div_magic);
    return g;
}

// One tile of channel (b, t): the records [r0, r1) of the example can reach it; cen is the
// grid centre.
// FUSED (small problems, index types): there are no records; the "records" [r0, r1) are the
// example's atoms themselves, and a lane transforms, culls and filters by type the atom it takes,
// with the arithmetic and the tests of the prep kernel.
template <bool BINARY, bool ALIGNED, int ITERS, int NW, typename OUT, bool FUSED = false>
__device__ __forceinline__ void tile_body(const FwdParams &p, float *lds, int b, int t,
                                          const TileGeom &tg, int r0, int r1, const float4 &cen)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const GridSpec &gs = p.gs;
    const int D = gs.D, T = p.T, N = p.N;
    const int total = D * D * D;
    const int f0 = tg.f0, f1 = tg.f1, R0 = tg.R0, R1 = tg.R1, i_lo = tg.i_lo, i_hi = tg.i_hi;
    TileCtx cx;
    cx.tile = lds;
    cx.marks = reinterpret_cast<unsigned char *>(lds + ITERS * 512) + wave * kTaskCap;
    cx.shared = reinterpret_cast<int *>(lds + ITERS * 512 + NW * (kTaskCap / 4));
    cx.lane = lane;
    cx.wave = wave;
    cx.D = D;
    cx.n = f1 - f0;
    cx.nrows = R1 - R0;
    cx.c0 = f0 - R0 * D;
    cx.c1 = f1 - 1 - (R1 - 1) * D;
    cx.rowA = 0;
    cx.rowB = 0;
    cx.res = gs.res;
    cx.inv_res = gs.inv_res;
    cx.g2k = p.g2k; cx.c2k = p.c2k; cx.sA = p.sA; cx.cA = p.cA;
    cx.debug = p.debug;

    OUT *dst = reinterpret_cast<OUT *>(p.out) + ((size_t)b * T + t) * (size_t)total + f0;
    cx.cen_x = cen.x;
    cx.cen_y = cen.y;
    cx.cen_z = cen.z;
    cx.hD = 0.5f * (float)(D - 1);
    const float ox = cx.cen_x - gs.half;
    cx.oy = cx.cen_y - gs.half;
    cx.oz = cx.cen_z - gs.half;

    const float4 *rec = p.rec + (size_t)b * N + r0;
    const int count = r1 - r0;
    if (count <= 0) {           // uniform: nothing can reach this tile
        store_tile<ALIGNED, ITERS, NW, OUT>(cx, dst, false, false);
        return;
    }
    Xform X;

    // How the wavefronts share the work: the `nsplit` wavefronts of a set take the atoms of
    // the span in turn (atom e goes to lane e / nsplit of member e % nsplit, round after
    // round) and every set works through the plane pairs pA0, pA0 + 2, ... pA1.  Usually
    // there is one set (all wavefronts, all pairs); four wavefronts on a tile with exactly
    // two plane pairs form two sets of two, one per pair.
    int nsplit = NW, sub = wave, pA0 = i_lo, pA1 = i_hi;
    if (NW == 4 && i_hi - i_lo >= 2 && i_hi - i_lo <= 3) {
        nsplit = 2;
        sub = wave & 1;
        pA0 = i_lo + 2 * (wave >> 1);
        pA1 = min(pA0 + 1, i_hi);
    }
    // FUSED: an atom's type, coordinates and radius are requested together (one trip to memory),
    // whatever the type turns out to be; finish_raw transforms, culls and filters by type with
    // the prep kernel's arithmetic and tests.
    struct RawAtom {
        int te;
        float cc[3], rad;
    };
    auto fetch_raw = [&](int base) {
        RawAtom ra;
        const int ec = min(base + lane * nsplit + sub, count - 1);      // count >= 1 here
        ra.te = p.raw.types[(size_t)b * N + ec];
        const float *c3 = p.raw.coords + ((size_t)b * N + ec) * 3;
        ra.cc[0] = c3[0]; ra.cc[1] = c3[1]; ra.cc[2] = c3[2];
        ra.rad = p.raw.radii[gs.radius_type_indexed ? (size_t)t : (size_t)b * N + ec];
        return ra;
    };
    auto finish_raw = [&](const RawAtom &ra, int e) {
        Atom at;
        at.a = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
        at.w = 1.0f;
        if (e < count && ra.te == t) {
            float pp[3];
            apply_xform(X, ra.cc, pp);
            const float r = gs.radius_scale * ra.rad;
            const float reach = BINARY ? r : r * gs.c;
            const float org[3] = {ox, cx.oy, cx.oz};
            const float span = (float)(D - 1) * gs.res, pad = 1.0e-3f * gs.res;
            bool live = (r > 0.0f) && (reach < 1.0e30f);
            for (int k = 0; k < 3; ++k)     // also false for NaN / infinite coordinates
                live = live && (pp[k] >= org[k] - reach - pad) && (pp[k] <= org[k] + span + reach + pad);
            if (live) at.a = make_float4(pp[0], pp[1], pp[2], r);
        }
        at.valid = at.a.w > 0.0f;
        return at;
    };
    auto load_atom = [&](int base) {
        const int e = base + lane * nsplit + sub;
        Atom at;
        at.a = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
        at.w = 1.0f;
        if (FUSED) return finish_raw(fetch_raw(base), e);
        if (e < count) at.a = rec[e];
        at.valid = (e < count) && (at.a.w > 0.0f);
        return at;
    };
    auto test_pair = [&](const Atom &at, int iA) {
        cx.rowA = iA * D - R0;
        cx.rowB = cx.rowA + D;
        const int jaA = max(-cx.rowA, 0), jbA = min(R1 - R0 - cx.rowA, D);
        const int jaB = max(-cx.rowB, 0), jbB = iA < i_hi ? min(R1 - R0 - cx.rowB, D) : 0;
        return pair_test<BINARY>(cx, p, at, ox, iA, jaA, jbA, jaB, jbB);
    };

    // the loads of the first round are under way; clear the tile meanwhile
    // (FUSED: the first atoms are requested before the pose is waited for and worked out)
    Atom at0;
    if (FUSED) {
        const RawAtom ra0 = fetch_raw(0);
        load_xform(X, b, p.raw.centers, p.raw.quats, p.raw.translations);
        at0 = finish_raw(ra0, lane * nsplit + sub);
    } else {
        at0 = load_atom(0);
    }
    {
        const float4 z4 = make_float4(0.0f, 0.0f, 0.0f, 0.0f);     // same bits as integer zeros
#pragma unroll
        for (int it = 0; it < 2 * ITERS / NW; ++it)
            reinterpret_cast<float4 *>(cx.tile)[it * 64 * NW + threadIdx.x] = z4;
        if (threadIdx.x < 2) cx.shared[threadIdx.x] = 0;
    }
    const bool single = count <= 64 * nsplit && pA1 - pA0 <= 1;    // one round, one pair of planes
    const int limit = (int)(kFixedLimit * 256.0f);
    bool any = false, fixed = !BINARY;
    if (NW == 1 && !single) {
        // One wavefront, several rounds: a single pass.  The tile starts in fixed point and
        // the bound on what can reach one voxel is kept up round by round; the moment it
        // passes the limit, the tile is turned into floats and stays so.  The records of
        // the next round are requested before this round's tasks run.
        int bound = 0;
        Atom at = at0;
        for (int base = 0; base < count; base += 64) {
            Atom next = at;
            if (base + 64 < count) next = load_atom(base + 64);
            for (int iA = pA0; iA <= pA1; iA += 2) {
                PairHit h = test_pair(at, iA);
                if (!BINARY && fixed) {
                    bound += min(pair_bound<false>(h, at), 1 << 24);
                    if (bound > limit) {
                        fixed = false;
                        for (int o = lane; o < ITERS * 512; o += 64)
                            cx.tile[o] = (float)reinterpret_cast<int *>(cx.tile)[o] * (1.0f / kFixedOne);
                        lds_sync();
                    }
                }
                any = pair_run<BINARY>(cx, h, fixed) || any;
            }
            at = next;
        }
    } else {
        PairHit h0;
        if (NW > 1) __syncthreads();                // shared[] is clear
        // pass 1: what can be added to one voxel at most decides fixed point or float (one
        // wavefront keeps the bound in a register, several add theirs up in LDS)
        // (index types: every record adds at most 1 to a voxel, so a short span needs no count)
        const bool short_span = count <= (int)kFixedLimit;
        int bound = 0;
        if (single) {
            h0 = test_pair(at0, pA0);
            if (!BINARY && !short_span) bound = pair_bound<false>(h0, at0);
        } else if (!BINARY && !short_span) {
            for (int base = 0; base < count && bound <= limit; base += 64 * nsplit) {
                const Atom at = base == 0 ? at0 : load_atom(base);
                for (int iA = pA0; iA <= pA1; iA += 2) {
                    const PairHit h = test_pair(at, iA);
                    bound += min(pair_bound<false>(h, at), 1 << 24);   // past the limit the value does not matter
                }
            }
        }
        if (NW > 1) {
            if (!short_span && lane == 0 && bound > 0) atomicAdd(&cx.shared[0], min(bound, 1 << 24));
            __syncthreads();                        // tile and shared[0] are ready
            if (!short_span) bound = cx.shared[0];
        }
        fixed = !BINARY && bound <= limit;
        // pass 2: the tasks
        if (single) {
            any = pair_run<BINARY>(cx, h0, fixed);
        } else {
            for (int base = 0; base < count; base += 64 * nsplit) {
                const Atom at = base == 0 ? at0 : load_atom(base);
                for (int iA = pA0; iA <= pA1; iA += 2) {
                    PairHit h = test_pair(at, iA);
                    any = pair_run<BINARY>(cx, h, fixed) || any;
                }
            }
        }
        if (NW > 1) {
            if (any && lane == 0) cx.shared[1] = 1;
            __syncthreads();                        // every wavefront's additions are in the tile
            any = cx.shared[1] != 0;
        }
    }
    store_tile<ALIGNED, ITERS, NW, OUT>(cx, dst, any, fixed);
}


// One workgroup per tile.  OUT: float, or double for a grid of doubles.
template <bool BINARY, bool ALIGNED, int ITERS, int NW, typename OUT, bool FUSED = false>
__global__ __launch_bounds__(64 * NW) void forward_kernel(FwdParams p)
{
    extern __shared__ __attribute__((aligned(16))) float lds[];   // tile | marks per wave | shared

    // Workgroup ids go round the 8 XCDs (id % 8), each with its own L2: runs of consecutive
    // tiles, which read the same atom records, can be given to one XCD.
    const GridSpec &gs = p.gs;
    const int D = gs.D, T = p.T, N = p.N;
    // Every kernel argument the preamble needs is fetched now, in one go, instead of in five
    // dependent trips to the scalar cache spread over the preamble: they are inputs of an
    // asm statement whose result (zero) enters the very first computation.  (Not `asm
    // volatile`: after one, the compiler no longer uses scalar loads for the spans.)
    unsigned zero;
    asm("s_mov_b32 %0, 0"
        : "=s"(zero)
        : "s"((unsigned long long)p.range), "s"((unsigned long long)p.rec),
          "s"((unsigned long long)p.gcen), "s"((unsigned long long)p.out), "s"(p.tiles_magic),
          "s"(p.t_magic), "s"(p.div_magic), "s"(p.tiles), "s"(p.pos_major), "s"(p.ka_chunks), "s"(p.ka_last), "s"(p.ka_shift), "s"(p.ka_skip), "s"(p.xcd_shift), "s"(p.n_remap), "s"(D),
          "s"(T), "s"(N), "s"(p.debug), "s"(gs.half));
    if (p.expect_tag != 0u && *p.tag != p.expect_tag) return;      // not the tables this call expects
    unsigned u = blockIdx.x + zero;
    if (p.xcd_shift >= 0 && u < p.n_remap) {
        const unsigned xcd = u & 7u, slot = u >> 3, sh = (unsigned)p.xcd_shift;
        u = ((slot >> sh) << (sh + 3)) + (xcd << sh) + (slot & ((1u << sh) - 1u));
    }
    // Keep-alive read: the tables the prep kernel wrote (records, spans, poses: a few MB) are read
    // example by example, so those of the later examples would lie untouched while hundreds of
    // MB of stores pass and be written back to HBM before their turn -- and a read that has to
    // come from HBM while the chip streams stores costs far more than its bytes.  Every
    // wavefront therefore also reads 1 KB of the tables, at a position scattered by its id
    // (the result is not used): every line is touched every few microseconds and stays cached.
    float4 ka = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
    if (p.ka_chunks) {
        const unsigned c = __umulhi((blockIdx.x + zero) * 2654435761u, p.ka_chunks);
        const unsigned off = min(c << p.ka_shift, p.ka_last) + ((threadIdx.x & 63u) << 4);
        if ((threadIdx.x & 63u) < (1u << (p.ka_shift - 4)) &&   // the chunk's lanes, 16 bytes each
            ((blockIdx.x + zero) & p.ka_skip) == 0u)            // (every wavefront, or one in 2, 4, 8)
            ka = *reinterpret_cast<const float4 *>(reinterpret_cast<const char *>(p.rec) + off);
    }
    const unsigned uq = div_u32(u, p.tiles_magic), ur = u - uq * p.tiles;
    const unsigned chan = p.pos_major ? ur : uq;
    const unsigned tile_in_chan = p.pos_major ? uq : ur;
    const int b = (int)div_u32(chan, p.t_magic);
    const int t = (int)chan - b * T;
    if (FUSED) {
        // small problems: no tables; the grid centre is the example's centre, the candidates are
        // the example's atoms (tile_body transforms and filters them)
        const TileGeom tgf = tile_geom<ITERS>(p, D, tile_in_chan);
        float4 cenf = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
        if (p.raw.centers) {
            cenf.x = p.raw.centers[3 * b];
            cenf.y = p.raw.centers[3 * b + 1];
            cenf.z = p.raw.centers[3 * b + 2];
        }
        int n = N;
        if (p.raw.natoms) {
            n = p.raw.natoms[b];
            n = n < 0 ? 0 : (n > N ? N : n);
        }
        tile_body<BINARY, ALIGNED, ITERS, NW, OUT, true>(p, lds, b, t, tgf, 0, n, cenf);
        return;
    }
    const size_t group = (size_t)b * T + t;
    // All the scalar loads of the preamble are issued together (one trip to L2, which is
    // slow while the chip streams stores): the span of records that can reach the planes
    // of the tile (counted from the example's first record) and the grid centre.
    const int2 *span = p.range + group * D;
    const float4 cen = *reinterpret_cast<const float4 *>(p.gcen + 4 * b);   // one 16-byte load
    const TileGeom tg = tile_geom<ITERS>(p, D, tile_in_chan);
    int r0 = 0, r1 = 0;
    if (!MG_DEBUG_IS(p, 3)) {   // timing aid 3: nothing but the zero stores
        r0 = span[tg.i_lo].x;
        r1 = span[tg.i_hi].y;
    }
    asm volatile("" ::"s"(r0), "s"(r1), "s"(cen.x), "s"(cen.y), "s"(cen.z));  // all in flight before the first wait
    if (MG_DEBUG_IS(p, 2)) r1 = r0;
    tile_body<BINARY, ALIGNED, ITERS, NW, OUT>(p, lds, b, t, tg, r0, r1, cen);
    asm volatile("" ::"v"(ka.x), "v"(ka.y), "v"(ka.z), "v"(ka.w));     // the keep-alive read is waited for here
}


// ---------------------------------------------------------------------------
// Vector types, real density: kVecGroup channels of one spatial tile per wavefront.
//
// Every atom feeds every channel, and the channels differ only in the radius that scales
// the distance (radii are looked up by type id) and in the atom's weight.  One pass over the
// atoms in reach of the tile therefore serves several channels: the records are loaded and
// tested against the tile's rows once, the tasks are staged once, and per voxel the squared
// distance x'^2 (in units of rmax/sqrt(k), rmax the widest radius of the group) is worked
// out once; channel q rescales it, x'^2_q = x'^2 (rmax/r_q)^2, evaluates its density and adds
// w_q rho_q into its own tile in LDS.  Beyond channel q's own cutoff rho_q is 0 by its
// formula, so the voxels of the widest sphere that a narrower one does not reach add nothing.
// The channels are taken in order of radius (chan_order, written by the prep kernel), so the
// spheres of a group are nearly the same size.
//   Gaussian  w exp2(-x'^2_q)          = sgn exp2(log2|w| - ratio2_q x'^2)
//   tail      w (sqrt(x'^2_q) sA - cA)^2 = sgn (s sqrt|w| sA ratio_q - sqrt|w| cA)^2,  s = sqrt(x'^2)
// log2|w|, sqrt|w| sA ratio_q and sqrt|w| cA are worked out once per atom (in the lane that
// holds the atom) and fetched by the lanes that walk its chords.
// ---------------------------------------------------------------------------
constexpr int kVecGroup = 4;

struct VecGroup {           // wave-uniform: the channels of this workgroup
    int chan[kVecGroup];        // channel index (for dead slots: any valid channel)
    bool live[kVecGroup];       // slot q holds a channel with a positive radius
    float ratio2[kVecGroup];    // (rmax / r_q)^2
    float sAq[kVecGroup];       // sA rmax / r_q
    float thq[kVecGroup];       // Gaussian region of channel q: x'^2 <= g^2 k / ratio2_q
    float r2[kVecGroup];        // binary mode: r_q * r_q (float, as the predicate's right-hand side)
    float rmax;
};

// Fixed-point tiles: sqrt(|w| rho) of a tail is at most sqrt(kFixedLimit) < 11 wherever the tail is
// used, so divided by kVecTailScale it lies in [0, 1] and the multiply-add's clamp (to [0, 1], free)
// replaces the min that cuts the tail off at the cutoff; the Gaussian's exponent carries the same
// factor (squared), and the conversion to fixed point multiplies it back.
constexpr float kVecTailScale = 16.0f;
static_assert(kVecTailScale * kVecTailScale >= kFixedLimit, "the scaled tail root must stay in [0, 1]");

struct VecAtom {            // per atom, per channel of the group (fixed point: see kVecTailScale)
    float lw[kVecGroup];        // log2 |w_q|  (-inf for w_q = 0: the Gaussian is then 0); fixed: - 8
    float su[kVecGroup];        // sqrt|w_q| sA ratio_q; fixed: / 16
    float sc[kVecGroup];        // sqrt|w_q| cA; fixed: / 16
    int neg;                    // bit q: w_q < 0  (binary mode: bit q: w_q > 0, the atom marks channel q)
};

// Run the staged tasks [0, ntasks): one (atom, row) chord per lane, kVecGroup channels per voxel.
// tiles: channel q's tile starts at cx.tile + q * stride floats.
template <bool FIXED, bool SIGNED>
__device__ inline void run_tasks_group(const TileCtx &cx, const VecGroup &vg, const Cand &cd,
                                       const VecAtom &va, int stride, int ntasks)
{
    int carry = 0;
    for (int base = 0; base < ntasks; base += 64) {
        const int tau = base + cx.lane;
        bool act = tau < ntasks;
        const int owner = max(carry, wave_inclusive_max((int)cx.marks[tau]));
        carry = bcast(owner, 63);
        const int src = (act ? owner - 1 : 0) << 2;
        const float fy = fetch(src, cd.c0), fz = fetch(src, cd.c1), stepk = fetch(src, cd.c2),
                    inv_stepk = fetch(src, cd.c3);
        const float pxA = fetch(src, cd.pxA), pxB = fetch(src, cd.pxB);
        const int pack = __builtin_amdgcn_ds_bpermute(src, cd.pack);
        const int k = tau - __builtin_amdgcn_ds_bpermute(src, cd.start);   // row number within the atom
        float lw[kVecGroup], su[kVecGroup], sc[kVecGroup];
#pragma unroll
        for (int q = 0; q < kVecGroup; ++q) {
            lw[q] = fetch(src, va.lw[q]);
            su[q] = fetch(src, va.su[q]);
            sc[q] = fetch(src, va.sc[q]);
        }
        int sb[kVecGroup];
        if (SIGNED) {
            const int neg = __builtin_amdgcn_ds_bpermute(src, va.neg);
#pragma unroll
            for (int q = 0; q < kVecGroup; ++q) sb[q] = ((neg >> q) & 1) << 31;
        }
        const int nA = (pack >> 10) & 1023;
        const bool inB = k >= nA;
        const int j = inB ? (pack >> 20) + (k - nA) : (pack & 1023) + k;   // row in its plane
        const int trow = (inB ? cx.rowB : cx.rowA) + j;                    // row in the tile
        const float px2 = inB ? pxB : pxA;                                 // plane term of x'^2
        const int clip_lo = trow == 0 ? cx.c0 : 0;
        const int clip_hi = trow == cx.nrows - 1 ? cx.c1 : cx.D - 1;
        float *rowp = cx.tile + (trow * cx.D - cx.c0);
        const float dyk = (((float)j - cx.hD) - fy) * stepk;
        const float x2b = fmaf(dyk, dyk, px2);
        const float rem = cx.c2k - x2b;
        act = act && rem > 0.0f;
        const float hz = __builtin_amdgcn_sqrtf(fmaxf(rem, 0.0f)) * inv_stepk + 1.0e-3f;
        const float fzi = fz + cx.hD;                                       // as a grid index
        const int klo = max(clip_lo, (int)ceilf(fzi - hz));
        const int khi = min(clip_hi, (int)floorf(fzi + hz));
        const int nz = act ? khi - klo + 1 : 0;
        const float z0 = (((float)klo - cx.hD) - fz) * stepk;
        const float fnz = (float)nz;
        float *q0 = rowp + klo;
        for (float fi = 0.0f; fi < fnz; fi += 1.0f, ++q0) {
            const float zs = fmaf(fi, stepk, z0);
            const float x2 = fmaf(zs, zs, x2b);
            const float sx = __builtin_amdgcn_sqrtf(x2);
#pragma unroll
            for (int q = 0; q < kVecGroup; ++q) {
                const float e = __builtin_amdgcn_exp2f(fmaf(-vg.ratio2[q], x2, lw[q]));
                // FIXED: the atom's constants carry 1/kVecTailScale (see VecAtom), so that the tail's
                // root stays below 1 and the clamp of the multiply-add cuts it off at the cutoff
                const float u = FIXED ? __builtin_amdgcn_fmed3f(fmaf(-sx, su[q], sc[q]), 0.0f, 1.0f)
                                      : fminf(fmaf(sx, su[q], -sc[q]), 0.0f);
                float val = x2 <= vg.thq[q] ? e : u * u;                    // |w_q| rho_q, 0 beyond the cutoff
                if (SIGNED) val = __int_as_float(__float_as_int(val) | sb[q]);
                if (FIXED) {
                    // |val| 2^24 + 1/2, truncated: rounded to the nearest fixed-point step
                    const float half = SIGNED ? __int_as_float(0x3f000000 | sb[q]) : 0.5f;
                    __hip_atomic_fetch_add(reinterpret_cast<int *>(q0) + q * stride,
                                           (int)fmaf(val, kFixedOne * kVecTailScale * kVecTailScale, half),
                                           __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
                } else {
                    __hip_atomic_fetch_add(q0 + q * stride, val, __ATOMIC_RELAXED,
                                           __HIP_MEMORY_SCOPE_WORKGROUP);
                }
            }
        }
    }
    lds_sync();
}

// Binary occupancy for a group of channels: the chord of the widest sphere is walked once, d^2 is
// worked out once per voxel in the fixed float order of the predicate, and channel q is marked
// where the atom's weight is positive and d^2 <= r_q^2.
__device__ inline void run_tasks_group_binary(const TileCtx &cx, const VecGroup &vg, const Cand &cd,
                                              const VecAtom &va, int stride, int ntasks)
{
    int carry = 0;
    for (int base = 0; base < ntasks; base += 64) {
        const int tau = base + cx.lane;
        bool act = tau < ntasks;
        const int owner = max(carry, wave_inclusive_max((int)cx.marks[tau]));
        carry = bcast(owner, 63);
        const int src = (act ? owner - 1 : 0) << 2;
        const float ay = fetch(src, cd.c0), az = fetch(src, cd.c1), reach2 = fetch(src, cd.c3);
        const float pxA = fetch(src, cd.pxA), pxB = fetch(src, cd.pxB);
        const int pack = __builtin_amdgcn_ds_bpermute(src, cd.pack);
        const int k = tau - __builtin_amdgcn_ds_bpermute(src, cd.start);   // row number within the atom
        const int pos = __builtin_amdgcn_ds_bpermute(src, va.neg);         // channels the atom marks
        const int nA = (pack >> 10) & 1023;
        const bool inB = k >= nA;
        const int j = inB ? (pack >> 20) + (k - nA) : (pack & 1023) + k;   // row in its plane
        const int trow = (inB ? cx.rowB : cx.rowA) + j;                    // row in the tile
        const float px2 = inB ? pxB : pxA;                                 // dx^2
        const int clip_lo = trow == 0 ? cx.c0 : 0;
        const int clip_hi = trow == cx.nrows - 1 ? cx.c1 : cx.D - 1;
        float *rowp = cx.tile + (trow * cx.D - cx.c0);
        const float gy = cx.oy + (float)j * cx.res;
        const float dy = gy - ay;
        const float dy2 = dy * dy;
        const float rem = (reach2 - px2) - dy2;
        act = act && rem > 0.0f;
        const float hz = __builtin_amdgcn_sqrtf(fmaxf(rem, 0.0f)) * cx.inv_res + 1.0e-3f;
        const float fz = (az - cx.oz) * cx.inv_res;
        const int klo = max(clip_lo, (int)ceilf(fz - hz));
        const int khi = min(clip_hi, (int)floorf(fz + hz));
        const int nz = act ? khi - klo + 1 : 0;
        const float base2 = px2 + dy2;
        for (int i = 0; i < nz; ++i) {
            const float gz = cx.oz + (float)(klo + i) * cx.res;
            const float dz = gz - az;
            const float d2 = base2 + dz * dz;
#pragma unroll
            for (int q = 0; q < kVecGroup; ++q)
                if (((pos >> q) & 1) && d2 <= vg.r2[q]) rowp[klo + i + q * stride] = 1.0f;
        }
    }
    lds_sync();
}

// Stage the tasks of the hits and run them (as pair_run, for a group of channels).
template <bool BINARY, bool SIGNED>
__device__ inline bool pair_run_group(const TileCtx &cx, const VecGroup &vg, PairHit &h,
                                      const VecAtom &va, int stride, bool fixed)
{
    int todo = h.nA + h.nB;
    if (__ballot(todo > 0) == 0ull) return false;
    while (true) {
        const int incl = wave_inclusive_scan(todo);
        int total = bcast(incl, 63);
        if (total == 0) break;
        bool now = todo > 0;
        if (total > kTaskCap) {     // rare: the rest waits for the next round
            now = now && incl <= kTaskCap;
            total = bcast(wave_inclusive_scan(now ? todo : 0), 63);
            if (total == 0) break;
        }
        if (cx.lane < kTaskCap / 16)
            reinterpret_cast<float4 *>(cx.marks)[cx.lane] = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
        if (now) {
            h.cd.start = incl - todo;
            cx.marks[h.cd.start] = (unsigned char)(cx.lane + 1);
            todo = 0;
        }
        lds_sync();
        if (BINARY) run_tasks_group_binary(cx, vg, h.cd, va, stride, total);
        else if (fixed) run_tasks_group<true, SIGNED>(cx, vg, h.cd, va, stride, total);
        else run_tasks_group<false, SIGNED>(cx, vg, h.cd, va, stride, total);
    }
    return true;
}

// One workgroup of NW wavefronts per (example, group of kVecGroup channels, tile).  The
// wavefronts share the group's tiles in LDS and take the rounds of 64 records in turn; every
// wavefront stages and runs its own tasks.  The tiles accumulate in fixed point; the bound on
// what can reach one voxel is summed up on the way, and a workgroup whose bound passes the
// limit at the end (rare) starts over in floats, all records taken by its first wavefront so
// that the order of the float additions is the same in every run.
template <bool BINARY, bool ALIGNED, int ITERS, int NW, typename OUT>
__global__ __launch_bounds__(64 * NW) void forward_vector_kernel(FwdParams p)
{
    extern __shared__ __attribute__((aligned(16))) float lds[];   // kVecGroup tiles | marks per wave | bound
    constexpr int kTile = ITERS * 512;
    const GridSpec &gs = p.gs;
    const int D = gs.D, T = p.T, N = p.N;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    if (p.expect_tag != 0u && *p.tag != p.expect_tag) return;      // not the tables this call expects
    const unsigned u = blockIdx.x;
    const unsigned uq = div_u32(u, p.tiles_magic), tile_in_chan = u - uq * p.tiles;
    const int b = (int)div_u32(uq, p.t_magic);          // t_magic: ceil(2^64 / groups)
    const int g = (int)uq - b * (int)p.groups;
    const int2 *span = p.range + (size_t)b * T * D;     // vector types: one record list per example
    const float4 cen = *reinterpret_cast<const float4 *>(p.gcen + 4 * b);
    const TileGeom tg = tile_geom<ITERS>(p, D, tile_in_chan);
    const int r0 = span[tg.i_lo].x, r1 = span[tg.i_hi].y;

    // the channels of this group and what depends on their radii only
    VecGroup vg;
    vg.rmax = 0.0f;
    float rq[kVecGroup];
#pragma unroll
    for (int q = 0; q < kVecGroup; ++q) {
        const int pos = g * kVecGroup + q;
        vg.chan[q] = p.chan_order[(size_t)b * T + min(pos, T - 1)];
        rq[q] = gs.radius_scale * p.radii[vg.chan[q]];
        vg.live[q] = pos < T && rq[q] > 0.0f && rq[q] < 1.0e30f;
        if (vg.live[q]) vg.rmax = fmaxf(vg.rmax, rq[q]);
    }
#pragma unroll
    for (int q = 0; q < kVecGroup; ++q) {
        const float ratio = vg.live[q] ? vg.rmax * __builtin_amdgcn_rcpf(rq[q]) : 1.0f;
        vg.ratio2[q] = ratio * ratio;
        vg.sAq[q] = p.sA * ratio;
        vg.thq[q] = p.g2k * __builtin_amdgcn_rcpf(vg.ratio2[q]);
        vg.r2[q] = vg.live[q] ? rq[q] * rq[q] : -1.0f;     // (nothing is within a dead channel's radius)
    }

    TileCtx cx;
    cx.tile = lds;
    cx.marks = reinterpret_cast<unsigned char *>(lds + kVecGroup * kTile) + wave * kTaskCap;
    cx.shared = reinterpret_cast<int *>(lds + kVecGroup * kTile + NW * (kTaskCap / 4));
    cx.lane = lane;
    cx.wave = wave;
    cx.D = D;
    cx.n = tg.f1 - tg.f0;
    cx.nrows = tg.R1 - tg.R0;
    cx.c0 = tg.f0 - tg.R0 * D;
    cx.c1 = tg.f1 - 1 - (tg.R1 - 1) * D;
    cx.rowA = 0;
    cx.rowB = 0;
    cx.res = gs.res;
    cx.inv_res = gs.inv_res;
    cx.g2k = p.g2k; cx.c2k = p.c2k; cx.sA = p.sA; cx.cA = p.cA;
    cx.debug = 0;
    cx.cen_x = cen.x; cx.cen_y = cen.y; cx.cen_z = cen.z;
    cx.hD = 0.5f * (float)(D - 1);
    const float ox = cx.cen_x - gs.half;
    cx.oy = cx.cen_y - gs.half;
    cx.oz = cx.cen_z - gs.half;

    const size_t total = (size_t)D * D * D;
    OUT *out = reinterpret_cast<OUT *>(p.out);
    auto store_all = [&](bool touched, bool fixed) {
#pragma unroll
        for (int q = 0; q < kVecGroup; ++q) {
            if (g * kVecGroup + q >= T) break;              // uniform
            TileCtx cq = cx;
            cq.tile = lds + q * kTile;
            OUT *dst = out + ((size_t)b * T + vg.chan[q]) * total + tg.f0;
            store_tile<ALIGNED, ITERS, NW, OUT>(cq, dst, touched && vg.live[q], fixed);
        }
    };
    const int count = r1 - r0;
    if (count <= 0 || !(vg.rmax > 0.0f)) {      // uniform: nothing can reach these tiles
        store_all(false, false);
        return;
    }

    const float4 *rec = p.rec + (size_t)b * N + r0;
    const int *idx = p.idx + (size_t)b * N + r0;
    const float *wbase = p.weights + (size_t)source_example(p.subgrids, b) * N * T;
    struct Raw {
        float4 a;
        int ai;
    };
    auto load_raw = [&](int base) {
        Raw r;
        r.a = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
        r.ai = 0;
        if (base + lane < count) {
            r.a = rec[base + lane];
            r.ai = idx[base + lane];
        }
        return r;
    };
    struct Wq {
        float w[kVecGroup];
    };
    auto gather = [&](const Raw &r) {
        Wq o;
        const float *row = wbase + (size_t)r.ai * T;
#pragma unroll
        for (int q = 0; q < kVecGroup; ++q)
            o.w[q] = (r.a.w > 0.0f && vg.live[q]) ? row[vg.chan[q]] : 0.0f;
        return o;
    };
    auto clear_tiles = [&]() {
        const float4 z4 = make_float4(0.0f, 0.0f, 0.0f, 0.0f);     // same bits as integer zeros
#pragma unroll
        for (int it = 0; it < kVecGroup * kTile / (256 * NW); ++it)
            reinterpret_cast<float4 *>(lds)[it * 64 * NW + threadIdx.x] = z4;
        if (threadIdx.x < 2) cx.shared[threadIdx.x] = 0;
    };

    // One pass over the rounds first, first + stride, ...: returns whether any task ran; adds
    // what the hits can put into one voxel at most to `bound` (1/256 units).  Records and
    // indices are requested two rounds ahead, the weights (gathered through the indices) one
    // round ahead; clear_first: the tiles are cleared while the first loads are in flight.
    auto pass = [&](int first, int stride, bool fixed, bool clear_first, int &bound) {
        bool any = false;
        Raw rc = load_raw(64 * first);
        Raw rn = load_raw(64 * (first + stride));
        Wq wc = gather(rc);
        if (clear_first) {
            clear_tiles();
            if (NW > 1) __syncthreads();
        }
        Wq wn = gather(rn);
        for (int base = 64 * first; base < count; base += 64 * stride) {
            const Raw rnn = load_raw(base + 128 * stride);
            // this round's atom: what its chords will need, per channel
            Atom at;
            at.a = rc.a;
            float wmax = 0.0f;
            VecAtom va;
            va.neg = 0;
#pragma unroll
            for (int q = 0; q < kVecGroup; ++q) {
                if (BINARY) {       // the atom marks the channels where its weight is positive
                    va.lw[q] = 0.0f; va.su[q] = 0.0f; va.sc[q] = 0.0f;
                    va.neg |= (wc.w[q] > 0.0f ? 1 : 0) << q;
                    continue;
                }
                const float aw = fabsf(wc.w[q]);
                wmax = fmaxf(wmax, aw);
                const float sw = __builtin_amdgcn_sqrtf(aw) * (fixed ? 1.0f / kVecTailScale : 1.0f);
                va.lw[q] = __builtin_amdgcn_logf(aw) - (fixed ? 8.0f : 0.0f);       // log2; 8 = log2 of the scale squared
                va.su[q] = sw * vg.sAq[q];
                va.sc[q] = sw * cx.cA;
                va.neg |= (wc.w[q] < 0.0f ? 1 : 0) << q;
            }
            at.w = wmax;
            at.valid = (rc.a.w > 0.0f) && (BINARY ? va.neg != 0 : wmax > 0.0f);
            at.a.w = vg.rmax;
            const bool any_neg = !BINARY && __ballot(at.valid && va.neg != 0) != 0ull;
            for (int iA = tg.i_lo; iA <= tg.i_hi; iA += 2) {
                cx.rowA = iA * D - tg.R0;
                cx.rowB = cx.rowA + D;
                const int jaA = max(-cx.rowA, 0), jbA = min(tg.R1 - tg.R0 - cx.rowA, D);
                const int jaB = max(-cx.rowB, 0), jbB = iA < tg.i_hi ? min(tg.R1 - tg.R0 - cx.rowB, D) : 0;
                PairHit h = pair_test<BINARY>(cx, p, at, ox, iA, jaA, jbA, jaB, jbB);
                if (!BINARY) bound = min(bound + min(pair_bound<true>(h, at), 1 << 24), 1 << 26);
                const bool ran = any_neg ? pair_run_group<BINARY, true>(cx, vg, h, va, kTile, fixed)
                                         : pair_run_group<BINARY, false>(cx, vg, h, va, kTile, fixed);
                any = ran || any;
            }
            rc = rn;
            wc = wn;
            rn = rnn;
            wn = gather(rn);
        }
        return any;
    };

    const int limit = (int)(kFixedLimit * 256.0f);
    int bound = 0;
    bool fixed = !BINARY;       // (binary tiles hold 0.0f / 1.0f as they are)
    bool any = pass(wave, NW, fixed, true, bound);
    if (NW > 1) {
        if (lane == 0) {
            atomicAdd(&cx.shared[0], bound);
            if (any) cx.shared[1] = 1;
        }
        __syncthreads();                    // every wavefront's additions are in the tiles
        bound = cx.shared[0];
        any = cx.shared[1] != 0;
    }
    if (!BINARY && bound > limit) {         // uniform over the workgroup: the sums may not fit; again, in floats
        if (NW > 1) __syncthreads();        // shared[] has been read by all
        fixed = false;
        clear_tiles();
        if (NW > 1) __syncthreads();
        int unused = 0;
        if (wave == 0) pass(0, 1, false, false, unused);
        if (NW > 1) __syncthreads();
    }
    store_all(any, fixed);
}

}  // namespace

ForwardGeometry forward_geometry(int D, int tile_floats)
{
    ForwardGeometry fg;
    fg.tile_floats = tile_floats;
    const long long total = (long long)D * D * D;
    fg.tiles = (int)((total + tile_floats - 1) / tile_floats);
    return fg;
}

namespace {
unsigned long long magic64(unsigned d)      // ceil(2^64 / d); 0 stands for d == 1
{
    if (d <= 1) return 0ull;
    const unsigned long long q = ~0ull / d;             // floor((2^64 - 1) / d)
    return q + 1ull;        // = ceil(2^64 / d): d >= 2 never divides 2^64 - 1 and 2^64 both, and
                            // when d divides 2^64, q = 2^64/d - 1
}
}  // namespace

// Vector types (real density and binary occupancy): one workgroup per (example, group of kVecGroup
// channels, tile).
static hipError_t launch_forward_vector(const GridSpec &gs, const Batch &bt, const Workspace &ws,
                                        void *out, bool out_is_double, int tile_floats,
                                        int waves_per_tile, unsigned expect_tag, KernelEvents ev,
                                        hipStream_t stream)
{
    // 2048-float tiles and four wavefronts per workgroup: the four channel tiles of a group take
    // 33 KB of LDS, so four workgroups (sixteen wavefronts, what 111 registers allow) fit a CU.
    // Measured on the 48^3 batch of 50 x 2040 atoms x 28 channels: 0.50 ms; relative to it, 1024
    // floats x 2 wavefronts +10 % (each tile tests the atoms in reach anew), 2048 x 2 and 1024 x 1
    // +43 % (too few wavefronts), 512 x 1 +33 %.  A grid of doubles takes 512 voxels per tile.
    if (tile_floats != 512 && tile_floats != 1024 && tile_floats != 2048) tile_floats = 2048;
    if (out_is_double) tile_floats = 512;
    const ForwardGeometry fg = forward_geometry(gs.D, tile_floats);
    FwdParams p;
    p.gs = gs;
    p.rec = ws.rec;
    p.idx = ws.idx;
    p.range = ws.range;
    p.weights = bt.weights;
    p.radii = bt.radii;
    p.gcen = ws.gcen;
    p.chan_order = ws.chan_order;
    p.tag = ws.tag;
    p.expect_tag = expect_tag;
    p.raw = RawInputs{};
    p.groups = (unsigned)((bt.T + kVecGroup - 1) / kVecGroup);
    p.out = out;
    p.subgrids = bt.sub.count; p.N = bt.N; p.T = bt.T;
    p.tile_floats = fg.tile_floats;
    p.div_magic = ((1ULL << 40) + (unsigned long long)gs.D - 1ULL) / (unsigned long long)gs.D;
    p.pos_major = 0u;
    p.tiles = (unsigned)fg.tiles;
    p.tiles_magic = magic64(p.tiles);
    p.t_magic = magic64(p.groups);
    p.xcd_shift = -1;
    p.n_remap = 0;
    p.debug = 0;
    p.ka_chunks = 0;
    p.ka_last = 0;
    p.ka_shift = 8;
    p.ka_skip = 0;
    const double k = 2.8853900817779268;        // 2 / ln 2
    p.sk = (float)std::sqrt(k);
    p.inv_sk = (float)(1.0 / std::sqrt(k));
    p.g2k = (float)((double)gs.g2 * k);
    p.c2k = (float)((double)gs.c * (double)gs.c * k);
    p.sA = (float)std::sqrt((double)gs.A / k);
    p.cA = (float)((double)gs.c * std::sqrt((double)gs.A));
    const unsigned long long wgs = (unsigned long long)bt.B * p.groups * fg.tiles;
    if (wgs > 0x7fffffffULL) return hipErrorInvalidValue;
    // four wavefronts per workgroup by default: they share the tiles, so four times as many
    // wavefronts are resident for the same LDS (the kernel is bound by vector arithmetic and
    // needs them to keep the SIMDs busy)
    int nw = waves_per_tile == 0 ? 4 : waves_per_tile;
    if (tile_floats == 512 || out_is_double) nw = 1;
    if (nw > tile_floats / 512) nw = tile_floats / 512;
    const size_t lds_bytes = (size_t)kVecGroup * tile_floats * sizeof(float) + (size_t)nw * kTaskCap + 16;
    const bool aligned = (gs.D % 4 == 0) && (((uintptr_t)out & 15u) == 0);
    const dim3 blk(64 * nw), grd((unsigned)wgs);
#define MG_VEC(Al, It, Nw, Ot)                                                                        \
    do {                                                                                              \
        if (gs.binary)                                                                                \
            hipExtLaunchKernelGGL((forward_vector_kernel<true, Al, It, Nw, Ot>), grd, blk,            \
                                  (uint32_t)lds_bytes, stream, ev.start, ev.stop, 0, p);              \
        else                                                                                          \
            hipExtLaunchKernelGGL((forward_vector_kernel<false, Al, It, Nw, Ot>), grd, blk,           \
                                  (uint32_t)lds_bytes, stream, ev.start, ev.stop, 0, p);              \
    } while (0)
#define MG_VEC_NW(Al, It, Ot) \
    if (nw == 1) MG_VEC(Al, It, 1, Ot); else MG_VEC(Al, It, 2, Ot)
    if (out_is_double) {
        if (aligned) MG_VEC(true, 1, 1, double); else MG_VEC(false, 1, 1, double);
    } else if (tile_floats == 512) {
        if (aligned) MG_VEC(true, 1, 1, float); else MG_VEC(false, 1, 1, float);
    } else if (tile_floats == 1024) {
        if (aligned) { MG_VEC_NW(true, 2, float); } else { MG_VEC_NW(false, 2, float); }
    } else if (nw == 4) {
        if (aligned) MG_VEC(true, 4, 4, float); else MG_VEC(false, 4, 4, float);
    } else {
        if (aligned) { MG_VEC_NW(true, 4, float); } else { MG_VEC_NW(false, 4, float); }
    }
#undef MG_VEC_NW
#undef MG_VEC
    return hipGetLastError();
}

bool forward_takes_single_launch(const Batch &bt, bool out_is_double)
{
    // index types into a float grid, no subgrids, at most kSmallAtoms atoms per example and
    // kSmallTotal in all: every tile's wavefront can afford to look at all of them itself
    return !bt.vec && !out_is_double && bt.sub.count == 1 && bt.N <= kSmallAtoms &&
           (long long)bt.B * bt.N <= kSmallTotal;
}

hipError_t launch_forward(const GridSpec &gs, const Batch &bt, const Workspace &ws, void *out,
                          bool out_is_double, int tile_floats, int waves_per_tile, int xcd_run,
                          int lds_floor, int debug, int tile_order, int keep_alive, bool single_launch,
                          unsigned expect_tag, KernelEvents ev, hipStream_t stream, int keep_alive_stride)
{
    if (bt.vec)
        return launch_forward_vector(gs, bt, ws, out, out_is_double, tile_floats, waves_per_tile, expect_tag, ev,
                                     stream);
    if (tile_floats == 512) tile_floats = 1024;     // the smallest tile of these kernels
    if (waves_per_tile == 0) waves_per_tile = 1;
    if (single_launch) {        // one shape only: 4 KB tiles, one wavefront, ids in order
        tile_floats = 1024;
        waves_per_tile = 1;
        xcd_run = 0;
        tile_order = 0;
        keep_alive = 0;
        lds_floor = 0;
    }
    if (tile_floats == 0) {
        // 4 KB tiles unless a tile meets many records (then the fixed cost per tile counts for
        // more than the shorter life of a small tile): about N/T atoms per channel, of which
        // those within a cutoff sphere's width (taken as 6 A) of the tile's x-plane are read.
        // Measured: 48^3 at 0.5 A with 2040 atoms (20 per tile) 102 us against 111 us with 8 KB
        // tiles; 96^3 at 0.25 A with 8000 atoms (74 per tile) 275 us with 8 KB tiles against 297 us,
        // with 6000 atoms (56 per tile) 281 against 279 us, with 5000 (47) 285 against 275 us.
        const double groups = bt.vec ? 1.0 : (double)bt.T;
        const double planes = 6.0 / (double)gs.res + 1.0;
        const double per_tile = (double)bt.N / groups * (planes < gs.D ? planes / gs.D : 1.0);
        tile_floats = per_tile > 60.0 ? 2048 : 1024;
        if (waves_per_tile > tile_floats / 512) waves_per_tile = tile_floats / 512;
    }
    if (out_is_double) {        // 512 voxels = 4 KB of doubles per one-wavefront workgroup
        tile_floats = 512;
        waves_per_tile = 1;
    }
    const ForwardGeometry fg = forward_geometry(gs.D, tile_floats);
    FwdParams p;
    p.gs = gs;
    p.rec = ws.rec;
    p.idx = ws.idx;
    p.range = ws.range;
    p.weights = bt.weights;
    p.radii = bt.radii;
    p.gcen = ws.gcen;
    p.chan_order = ws.chan_order;
    p.tag = ws.tag;
    p.expect_tag = single_launch ? 0u : expect_tag;
    p.groups = 0;
    p.raw.coords = bt.coords; p.raw.types = bt.types; p.raw.radii = bt.radii; p.raw.natoms = bt.natoms;
    p.raw.centers = bt.centers; p.raw.quats = bt.quats; p.raw.translations = bt.translations;
    p.out = out;
    p.subgrids = bt.sub.count; p.N = bt.N; p.T = bt.T;
    p.tile_floats = fg.tile_floats;
    p.div_magic = ((1ULL << 40) + (unsigned long long)gs.D - 1ULL) / (unsigned long long)gs.D;
    const int iters = tile_floats / 512;
    int nw = waves_per_tile < iters ? waves_per_tile : iters;
    if (iters == 8 && nw < 2) nw = 2;           // 16 KB tiles are built for two or four wavefronts
    p.pos_major = tile_order == 1 ? 1u : 0u;
    p.tiles = p.pos_major ? (unsigned)bt.B * (unsigned)bt.T : (unsigned)fg.tiles;
    p.tiles_magic = magic64(p.tiles);
    p.t_magic = magic64((unsigned)bt.T);
    const unsigned long long groups = (unsigned long long)bt.B * bt.T * fg.tiles;
    p.xcd_shift = -1;
    p.n_remap = 0;
    for (int sh = 0; sh < 16; ++sh)
        if (xcd_run == (1 << sh)) p.xcd_shift = sh;
    if (p.xcd_shift >= 0) {
        const unsigned long long chunk = 8ull << p.xcd_shift;
        p.n_remap = (unsigned)(groups / chunk * chunk);
    }
    p.debug = debug;
    {   // the tables lie one after the other in the workspace, from the records to the grid centres
        const size_t bytes = (size_t)((const char *)(ws.gcen + (size_t)bt.B * 4) - (const char *)ws.rec);
        p.ka_chunks = 0;
        p.ka_last = 0;
        p.ka_skip = keep_alive_stride > 1 ? (unsigned)keep_alive_stride - 1u : 0u;
        // keep_alive: 0 = none, 1 = the default chunk, else the chunk in bytes (256, 512, 1024)
        const unsigned chunk = keep_alive == 1 ? kKeepAliveBytes : (unsigned)keep_alive;
        p.ka_shift = chunk == 1024u ? 10u : (chunk == 512u ? 9u : (chunk == 128u ? 7u : (chunk == 64u ? 6u : 8u)));
        // (vector types are bound by arithmetic and a grid of doubles by its own stores: measured no gain)
        if (keep_alive && !bt.vec && !out_is_double && bytes >= 1024 && bytes < (1ull << 31)) {
            p.ka_chunks = (unsigned)((bytes + chunk - 1) >> p.ka_shift);
            p.ka_last = (unsigned)(bytes - chunk);
        }
    }
    const double k = 2.8853900817779268;        // 2 / ln 2
    p.sk = (float)std::sqrt(k);
    p.inv_sk = (float)(1.0 / std::sqrt(k));
    p.g2k = (float)((double)gs.g2 * k);
    p.c2k = (float)((double)gs.c * (double)gs.c * k);
    p.sA = (float)std::sqrt((double)gs.A / k);
    p.cA = (float)((double)gs.c * std::sqrt((double)gs.A));
    // tile | marks of each wavefront | shared words; lds_floor raises the request to cap how
    // many tiles are resident on a CU
    size_t lds_bytes = (size_t)tile_floats * sizeof(float) + (size_t)nw * kTaskCap + 16;
    // 4 KB tiles, one wavefront each: 26 per CU (104 KB of stores in flight) instead of all 32
    // slots measured 98.2 us against 102.4 us on the 48^3 batch (22 to 30 per CU alike)
    if (lds_floor < 0) lds_floor = (tile_floats == 1024 && nw == 1 && !out_is_double && !bt.vec) ? 6144 : 0;
    if (lds_bytes < (size_t)lds_floor) lds_bytes = (size_t)lds_floor;
    const bool aligned = (gs.D % 4 == 0) && (((uintptr_t)out & 15u) == 0);
    const dim3 blk(64 * nw), grd((unsigned)groups);
#define MG_LAUNCH5(Bn, Al, It, Nw) \
    hipExtLaunchKernelGGL((forward_kernel<Bn, Al, It, Nw, float>), grd, blk, (uint32_t)lds_bytes, \
                          stream, ev.start, ev.stop, 0, p)
#define MG_LAUNCH(Bn, Al)                                                       \
    if (out_is_double) {                                                        \
        hipExtLaunchKernelGGL((forward_kernel<Bn, Al, 1, 1, double>), grd, blk,                    \
                              (uint32_t)lds_bytes, stream, ev.start, ev.stop, 0, p);               \
    } else switch (iters * 8 + nw) {                                            \
    case 2 * 8 + 1: MG_LAUNCH5(Bn, Al, 2, 1); break;                            \
    case 2 * 8 + 2: MG_LAUNCH5(Bn, Al, 2, 2); break;                            \
    case 4 * 8 + 1: MG_LAUNCH5(Bn, Al, 4, 1); break;                            \
    case 4 * 8 + 2: MG_LAUNCH5(Bn, Al, 4, 2); break;                            \
    case 4 * 8 + 4: MG_LAUNCH5(Bn, Al, 4, 4); break;                            \
    case 8 * 8 + 2: MG_LAUNCH5(Bn, Al, 8, 2); break;                            \
    case 8 * 8 + 4: MG_LAUNCH5(Bn, Al, 8, 4); break;                            \
    default: return hipErrorInvalidValue;                                       \
    }
    if (single_launch) {
#define MG_FUSED(Bn, Al) \
    hipExtLaunchKernelGGL((forward_kernel<Bn, Al, 2, 1, float, true>), grd, blk, (uint32_t)lds_bytes, \
                          stream, ev.start, ev.stop, 0, p)
        if (gs.binary) { if (aligned) MG_FUSED(true, true); else MG_FUSED(true, false); }
        else           { if (aligned) MG_FUSED(false, true); else MG_FUSED(false, false); }
#undef MG_FUSED
    } else {
        if (gs.binary) { if (aligned) MG_LAUNCH(true, true) else MG_LAUNCH(true, false) }
        else           { if (aligned) MG_LAUNCH(false, true) else MG_LAUNCH(false, false) }
    }
#undef MG_LAUNCH
#undef MG_LAUNCH5
    return hipGetLastError();
}

}  // namespace mg
