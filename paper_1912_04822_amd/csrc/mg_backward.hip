// Step 6 of the path: the backward pass (GridMaker section: "computes atomic
// gradients").  With L = sum G*out, u = x'_a - p, d = |u|, x = d/r:
//   dL/dx'_a = sum_p G[p] rho'(x) u / (r d)
//            = (1/r^2) sum_p G[p] f(x^2) u,
//   f = -4 exp(-2x^2)            x <= g      (rho' = -4x exp(-2x^2))
//     = 2A (1 - c/x)             g < x < c   (rho' = 2A (x - c))
//     = 0                        x >= c
// (dividing rho' by x removes the square root from the Gaussian branch and makes
// d = 0 contribute exactly 0 through u = 0).  The kernels sum -f/4 instead,
//   -f/4 = exp(-2x^2)            x <= g
//        = (A/2) (c/x - 1)       g < x < c     (at most exp(-2g^2) <= 1 there)
//        = 0                     x >= c
// which the hardware evaluates as one fused multiply-add clamped to [0,1] (the tail
// is <= 1 on its own interval and negative beyond the cutoff), and the factor -4 goes
// into the scale applied once per atom.  The gradient with respect to the caller's
// coordinates is R^T times that sum.
//
// One wavefront per atom record (four records per workgroup, no barrier).  The
// work items are "slots": runs of four voxels along z in the grid rows (x-plane,
// y) of the atom's cutoff box, read with one 16-byte load each.  Only the rows
// that meet the cutoff sphere are visited, and a row's slots start at the first
// voxel of its chord (so a chord of L voxels takes ceil(L/4) slots, wherever it
// lies; the last slot is pulled back into the row if need be -- voxels outside the
// sphere add exactly 0): per group of 128
// rows every lane works out the chord of its two rows, a prefix sum over
// the lanes numbers the live slots, and slot s finds its row through a byte
// array in LDS (the first slot of each lane's rows is marked with the lane, a
// running maximum over the slots gives the owner) and one register exchange.
// The kernel is bound by vector arithmetic (two transcendentals per voxel), so
// the time goes with the number of voxels evaluated.  The three partial sums
// are reduced across the wavefront by DPP adds in a fixed order.  Records are grouped by
// channel (and, within a channel, by x-plane), so neighbouring wavefronts read
// the same part of the same channel volume.
// (Consecutive lanes take consecutive slots of a row, so a 64-lane load touches about 25
// lines.  Two atoms per wavefront with every lane walking the slots of its own rows -- no
// slot list at all, a quarter fewer instructions -- touches 64 lines per load and measured
// 74-100 us against 62 us.)
#include <cmath>

#include "mg_common.h"
#include "mg_wave.h"

namespace mg {

namespace {

struct BwdParams {
    GridSpec gs;
    const float4 *rec;
    const int *idx;
    const int4 *meta;
    const float *rot;
    const int *rchan;       // [B][N] channel of each record (index types)
    const float *weights;
    const float *radii;
    const float *gcen;
    const unsigned char *alive;     // [B][N] 1: the atom has a live record
    const unsigned *tag;            // what the workspace's tables were made for
    unsigned expect_tag;            // != 0: do nothing unless *tag equals it (calls on prepared tables)
    const void *G;          // upstream gradient grid, float or double
    float *grad_coords;
    float *grad_weights;
    int subgrids, N, T;
    unsigned wgs_per_example;       // workgroups (of four records) per example
    unsigned units, share;          // workgroups in all; per XCD (ceil(units / 8))
    unsigned long long wg_magic;    // ceil(2^64 / wgs_per_example), 0 if that is 1
    float sk, inv_sk, g2k, c2k;     // sqrt(k), 1/sqrt(k), g^2 k, c^2 k with k = 2 log2(e)
    float hA, hAck;         // A/2, (A/2) c sqrt(k): -f/4 = clamp(hAck / x' - hA, 0, 1) in the tail
    float sAk, cA;          // sqrt(A/k), c sqrt(A)
};

// v + (v of the lane the DPP control selects, 0 where there is none or the row is masked out)
template <int CTRL, int ROW_MASK>
__device__ inline float add_dpp(float v)
{
    return v + __int_as_float(
                   __builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, ROW_MASK, 0xf, false));
}

// Sum over the 64 lanes in a fixed order (an inclusive scan by DPP row shifts and row
// broadcasts, whose last lane holds the total); returned in every lane.
__device__ inline float wave_sum(float v)
{
    v = add_dpp<0x111, 0xf>(v);     // row_shr:1
    v = add_dpp<0x112, 0xf>(v);     // row_shr:2
    v = add_dpp<0x114, 0xf>(v);     // row_shr:4
    v = add_dpp<0x118, 0xf>(v);     // row_shr:8
    v = add_dpp<0x142, 0xa>(v);     // row_bcast:15 -> rows 1, 3
    v = add_dpp<0x143, 0xc>(v);     // row_bcast:31 -> rows 2, 3
    return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 63));
}

struct Box {
    int ilo, jlo, seg0;
    int np, nr, ns;
    int klo, khi;
};

constexpr int kSlotCap = 1024;      // live slots of a group of 128 rows: at most 8 per row
constexpr int kMaxCulledSegs = 8;   // boxes with more z-segments per row take the plain loop
constexpr int kMaxCulledRows = 32768;   // ... and so do boxes with more rows: below that, row / nr by a
                                        // float reciprocal is exact (error <= rows * 2e-7 < 0.5)

// grid points within `reach` of the atom along each axis, padded by 1e-3 steps
__device__ inline bool atom_box(const GridSpec &gs, float reach, const float4 &a, float ox, float oy,
                                float oz, Box &bx)
{
    const float hv = reach * gs.inv_res + 1.0e-3f;
    const float fx = (a.x - ox) * gs.inv_res, fy = (a.y - oy) * gs.inv_res,
                fz = (a.z - oz) * gs.inv_res;
    const int D = gs.D;
    const int ilo = max(0, (int)ceilf(fx - hv)), ihi = min(D - 1, (int)floorf(fx + hv));
    const int jlo = max(0, (int)ceilf(fy - hv)), jhi = min(D - 1, (int)floorf(fy + hv));
    const int klo = max(0, (int)ceilf(fz - hv)), khi = min(D - 1, (int)floorf(fz + hv));
    bx.ilo = ilo; bx.jlo = jlo; bx.seg0 = klo >> 2; bx.klo = klo; bx.khi = khi;
    bx.np = ihi - ilo + 1; bx.nr = jhi - jlo + 1; bx.ns = (khi >> 2) - (klo >> 2) + 1;
    return bx.np > 0 && bx.nr > 0 && bx.ns > 0 && khi >= klo;
}

// Accumulate over one channel volume, in coordinates scaled to units of r/sqrt(k),
// k = 2 log2(e) (then exp(-2x^2) = exp2(-x'^2)):  (sx, sy, sz) += sum G (-f/4) u',  sv += sum G rho.
//   -f/4 = exp2(-x'^2)                                  x'^2 <= g^2 k
//        = clamp((A/2) c sqrt(k) / x' - A/2, 0, 1)      beyond (zero from the cutoff on)
// One slot: the four voxels k4 .. k4+3 of the grid row at float offset `row_off` of the
// channel (a channel has at most 2^30 floats); ux, uy: the row's scaled x and y distance.
struct SlotData {
    float gv[4];        // upstream gradient of the four voxels
    float ux, uy;
    int k4;
};

// 16-byte vectors that are only aligned like their elements (one wide load all the same)
typedef float Float4E __attribute__((ext_vector_type(4), aligned(4)));
typedef double Double2E __attribute__((ext_vector_type(2), aligned(8)));

// STREAM: the loads carry the non-temporal hint, so the lines they bring in do not settle in the
// memory-side cache.  The index-type kernel reads each line of the gradient grid once (its reuse
// is between neighbouring wavefronts, within microseconds, in L2), and the grid usually arrives
// behind hundreds of MB that an earlier kernel has just written and that still sit dirty in
// that cache: lines that settle there push those out, and the reads then wait behind the
// write-backs.  Measured on the 48^3 batch: 74 against 100 us right after a forward call, 74
// against 72 us after a read-only pass over another buffer, 71 against 62 us in a loop of
// nothing but backward calls (where the lines of the call before would otherwise still be
// cached).  The vector-typed kernel visits every line once per group of channels and atoms far
// apart in time share lines: with the hint it took 1.55 instead of 0.98 ms, so it goes without.
template <bool ALIGNED, bool STREAM, typename GT>
__device__ inline void load_slot(const BwdParams &p, const GT *Gc, unsigned row_off, int k4,
                                 float ux, float uy, SlotData &d)
{
    const GT *src = Gc + (row_off + (unsigned)k4);
    if (ALIGNED) {      // the four voxels lie in the row; k4 need not be a multiple of 4
        if (sizeof(GT) == 8) {      // a grid of doubles: two 16-byte loads, narrowed
            const Double2E *s2 = reinterpret_cast<const Double2E *>(src);
            const Double2E lo = STREAM ? __builtin_nontemporal_load(s2) : s2[0];
            const Double2E hi = STREAM ? __builtin_nontemporal_load(s2 + 1) : s2[1];
            d.gv[0] = (float)lo.x; d.gv[1] = (float)lo.y; d.gv[2] = (float)hi.x; d.gv[3] = (float)hi.y;
        } else {
            const Float4E *s4 = reinterpret_cast<const Float4E *>(src);
            const Float4E g4 = STREAM ? __builtin_nontemporal_load(s4) : *s4;
            d.gv[0] = g4.x; d.gv[1] = g4.y; d.gv[2] = g4.z; d.gv[3] = g4.w;
        }
    } else {
#pragma unroll
        for (int u = 0; u < 4; ++u)
            d.gv[u] = (k4 + u < p.gs.D) ? (float)(STREAM ? __builtin_nontemporal_load(src + u) : src[u]) : 0.0f;
    }
    d.ux = ux; d.uy = uy; d.k4 = k4;
}

template <bool WANT_VALUE>
__device__ inline void reduce_slot(const BwdParams &p, float step, float azs, const SlotData &d,
                                   float &sx, float &sy, float &sz, float &sv)
{
    const float ux = d.ux, uy = d.uy;
    const int k4 = d.k4;
    const float *gv = d.gv;
    const float b2 = ux * ux + uy * uy;
    const float uz0 = fmaf(-(float)k4, step, azs);
    float fsum = 0.0f;
#pragma unroll
    for (int u = 0; u < 4; ++u) {
        const float uz = uz0 - (float)u * step;
        const float x2 = fmaf(uz, uz, b2);
        const float e = __builtin_amdgcn_exp2f(-x2);
        const float rs = __builtin_amdgcn_rsqf(x2);
        const float ft = __builtin_amdgcn_fmed3f(fmaf(p.hAck, rs, -p.hA), 0.0f, 1.0f);
        const float f = x2 <= p.g2k ? e : ft;       // -f/4
        const float gf = gv[u] * f;
        fsum += gf;
        sz = fmaf(gf, uz, sz);
        if (WANT_VALUE) {
            const float tl = __builtin_amdgcn_fmed3f(fmaf(-(x2 * rs), p.sAk, p.cA), 0.0f, 1.0f);     // sqrt(A) (c - x), clamped to [0, 1]
            const float rho = x2 <= p.g2k ? e : tl * tl;
            sv = fmaf(gv[u], rho, sv);
        }
    }
    sx = fmaf(fsum, ux, sx);
    sy = fmaf(fsum, uy, sy);
}

// Every slot of the box (boxes with very many segments per row).
template <bool ALIGNED, bool WANT_VALUE, typename GT>
__device__ inline void reduce_channel_box(const BwdParams &p, const GT *Gc, const float4 &a,
                                          float r, const Box &bx, float ox, float oy, float oz,
                                          float &sx, float &sy, float &sz, float &sv)
{
    const GridSpec &gs = p.gs;
    const int per_plane = bx.nr * bx.ns;
    const int slots = bx.np * per_plane;        // at most D^3 / 4 < 2^31
    const float s = p.sk / r, step = gs.res * s;
    const float azs = (a.z - oz) * s;
    // scaled distance of the box's first row; rows step by `step`
    const float ux0 = (a.x - (ox + (float)bx.ilo * gs.res)) * s;
    const float uy0 = (a.y - (oy + (float)bx.jlo * gs.res)) * s;
    for (int sl = (int)(threadIdx.x & 63u); sl < slots; sl += 64) {
        // integer division: a box of hundreds of voxels per side has more slots than a float
        // holds exactly
        const int pi = sl / per_plane;
        const int rem = sl - pi * per_plane;
        const int row = rem / bx.ns;
        const int seg = rem - row * bx.ns;
        const float ux = fmaf(-(float)pi, step, ux0), uy = fmaf(-(float)row, step, uy0);
        SlotData d;
        load_slot<ALIGNED, false>(p, Gc, (unsigned)((bx.ilo + pi) * gs.D + bx.jlo + row) * (unsigned)gs.D,
                           (bx.seg0 + seg) << 2, ux, uy, d);
        reduce_slot<WANT_VALUE>(p, step, azs, d, sx, sy, sz, sv);
    }
}

// Only the slots that meet the cutoff sphere.  `marks` is this wavefront's kSlotCap bytes of
// LDS, all zero on entry and on return.
// The channel is G + t * D3 (index types: t comes with the record, from the workspace).
template <bool ALIGNED, bool WANT_VALUE, typename GT>
__device__ inline void reduce_channel(const BwdParams &p, const GT *G, int t, size_t D3,
                                      const float4 &a, float r, const Box &bx, float ox, float oy,
                                      float oz, unsigned char *marks, float &sx, float &sy,
                                      float &sz, float &sv)
{
    if (bx.ns > kMaxCulledSegs || bx.np * bx.nr > kMaxCulledRows) {
        reduce_channel_box<ALIGNED, WANT_VALUE>(p, G + (size_t)t * D3, a, r, bx, ox, oy, oz, sx, sy,
                                                sz, sv);
        return;
    }
    const GridSpec &gs = p.gs;
    const int lane = (int)(threadIdx.x & 63u);
    const int rows = bx.np * bx.nr;
    // reciprocals by the hardware approximation (1 ulp): the row split below has a margin of
    // 0.5/nr and the scale enters the result with a relative error of 1e-7
    const float inv_nr = __builtin_amdgcn_rcpf((float)bx.nr);
    const float s = p.sk * __builtin_amdgcn_rcpf(r), step = gs.res * s;
    const float inv_step = __builtin_amdgcn_rcpf(step);
    const float azs = (a.z - oz) * s;
    const float fz = (a.z - oz) * gs.inv_res;           // the atom's z in grid steps
    // scaled distance of the box's first row; rows step by `step`
    const float ux0 = (a.x - (ox + (float)bx.ilo * gs.res)) * s;
    const float uy0 = (a.y - (oy + (float)bx.jlo * gs.res)) * s;
    const unsigned D = (unsigned)gs.D;
    const unsigned off0 = ((unsigned)bx.ilo * D + (unsigned)bx.jlo) * D;   // the box's first row
    for (int row0 = 0; row0 < rows; row0 += 128) {
        // this lane's two rows of the group: which segments meet the sphere
        int cnt[2] = {0, 0}, slo[2] = {0, 0};
#pragma unroll
        for (int q = 0; q < 2; ++q) {
            const int row = row0 + 2 * lane + q;
            if (row < rows) {
                const int pi = (int)(((float)row + 0.5f) * inv_nr);
                const int jr = row - pi * bx.nr;
                const float ux = fmaf(-(float)pi, step, ux0), uy = fmaf(-(float)jr, step, uy0);
                const float h2 = p.c2k - (ux * ux + uy * uy);
                if (h2 > 0.0f) {
                    // half chord in grid steps; the pad only adds voxels that contribute 0
                    const float hv = __builtin_amdgcn_sqrtf(h2) * inv_step + 1.0e-3f;
                    const int klo = max(bx.klo, (int)ceilf(fz - hv));
                    const int khi = min(bx.khi, (int)floorf(fz + hv));
                    if (khi >= klo) {       // 4-voxel slots from the chord's first voxel, kept inside the row
                        cnt[q] = (khi - klo + 4) >> 2;
                        slo[q] = ALIGNED ? min(klo, gs.D - 4 * cnt[q]) : klo;
                    }
                }
            }
        }
        const int mine = cnt[0] + cnt[1];
        const int incl = wave_inclusive_scan(mine);
        const int total = bcast(incl, 63);
        const int excl = incl - mine;
        if (mine > 0) marks[excl] = (unsigned char)(lane + 1);
        // what a slot needs of its owner: first slot (11 bits) and slots of row 0 in one word,
        // the first voxel of row 0 and of row 1 (16 bits each) in another
        const int word = excl | (cnt[0] << 11), starts = slo[0] | (slo[1] << 16);
        lds_sync();
        asm volatile("" : "+v"(t));     // nothing above waits for t
        const GT *Gc = G + (size_t)t * D3;
        // Round k works on slots 64k .. 64k+63, one per lane.  (Issuing the reads of two or three
        // rounds before the arithmetic of the first was measured slower -- 69 against 62 us with
        // the gradient grid partly in the memory-side cache, 102 against 100 us with a grid that
        // has to come from HBM: the kernel fetches every 128-byte line of the gradient grid that
        // holds an in-cutoff voxel exactly once, 270 MB on the 48^3 batch, and runs at the rate
        // those scattered lines arrive, whatever the wavefronts have in flight.)
        int carry = 0;
        for (int base = 0; base < total; base += 64) {
            const int sidx = base + lane;
            int v = sidx < total ? (int)marks[sidx] : 0;
            v = max(wave_inclusive_max(v), carry);      // owner of slot 0 is marked: v >= 1
            carry = bcast(v, 63);
            const int owner = v - 1;
            const int w = __builtin_amdgcn_ds_bpermute(owner << 2, word);
            const int st = __builtin_amdgcn_ds_bpermute(owner << 2, starts);
            if (sidx < total) {
                const int o = sidx - (w & 0x7ff);
                const int c0 = w >> 11;
                const int q = o >= c0 ? 1 : 0;
                const int k4 = q ? (st >> 16) + 4 * (o - c0) : (st & 0xffff) + 4 * o;
                const int row = row0 + 2 * owner + q;
                const int pi = (int)(((float)row + 0.5f) * inv_nr);
                const int jr = row - pi * bx.nr;
                const float ux = fmaf(-(float)pi, step, ux0), uy = fmaf(-(float)jr, step, uy0);
                SlotData d;
                load_slot<ALIGNED, true>(p, Gc, off0 + ((unsigned)pi * D + (unsigned)jr) * D, k4, ux,
                                   uy, d);
                reduce_slot<WANT_VALUE>(p, step, azs, d, sx, sy, sz, sv);
            }
        }
        lds_sync();
        if (mine > 0) marks[excl] = 0;
        lds_sync();
    }
}

// ---------------------------------------------------------------------------
// Vector types: kChanGroup channels of one atom in one pass.  The channels differ only in
// radius, so the slots are listed once, for the widest sphere of the group (radius rmax),
// and every voxel's x'^2 (in units of rmax/sqrt(k)) is rescaled per channel:
//   x'^2_q = x'^2 (rmax/r_q)^2.   Beyond channel q's own cutoff f and rho are 0 by their
// formulas, so the voxels the narrower spheres do not reach add nothing.
// ---------------------------------------------------------------------------
constexpr int kChanGroup = 4;

struct GroupCoef {
    float ratio2[kChanGroup];       // (rmax / r_q)^2
    float cq[kChanGroup];           // -4 w_q rmax / (sqrt(k) r_q^2): channel q's share of the coordinate sums
    bool live[kChanGroup];          // r_q > 0 and t0 + q < T (uniform over the wavefront)
};

// body(row_off, k4, ux, uy) for every slot of the box that meets the sphere of radius r:
// the slot is the four voxels k4 .. k4+3 of the row at float offset row_off of a channel;
// ux, uy are the row's distances in units of r/sqrt(k).  The same enumeration as
// reduce_channel (marks: this wavefront's kSlotCap bytes of LDS, zero on entry and return).
template <bool ALIGNED, typename Body>
__device__ inline void for_each_slot(const BwdParams &p, const float4 &a, float r, const Box &bx,
                                     float ox, float oy, float oz, unsigned char *marks,
                                     Body body)
{
    const GridSpec &gs = p.gs;
    const int lane = (int)(threadIdx.x & 63u);
    const unsigned D = (unsigned)gs.D;
    const float s = p.sk * __builtin_amdgcn_rcpf(r), step = gs.res * s;
    const float ux0 = (a.x - (ox + (float)bx.ilo * gs.res)) * s;
    const float uy0 = (a.y - (oy + (float)bx.jlo * gs.res)) * s;
    const unsigned off0 = ((unsigned)bx.ilo * D + (unsigned)bx.jlo) * D;   // the box's first row
    if (bx.ns > kMaxCulledSegs || bx.np * bx.nr > kMaxCulledRows) {     // a very large box: every slot of it
        const int per_plane = bx.nr * bx.ns;
        const int slots = bx.np * per_plane;        // at most D^3 / 4 < 2^31
        for (int sl = lane; sl < slots; sl += 64) {
            const int pi = sl / per_plane;          // integer division: exact for any box
            const int rem = sl - pi * per_plane;
            const int row = rem / bx.ns;
            const int seg = rem - row * bx.ns;
            body(off0 + ((unsigned)pi * D + (unsigned)row) * D, (bx.seg0 + seg) << 2,
                 fmaf(-(float)pi, step, ux0), fmaf(-(float)row, step, uy0));
        }
        return;
    }
    const int rows = bx.np * bx.nr;
    const float inv_nr = __builtin_amdgcn_rcpf((float)bx.nr);
    const float inv_step = __builtin_amdgcn_rcpf(step);
    const float fz = (a.z - oz) * gs.inv_res;           // the atom's z in grid steps
    for (int row0 = 0; row0 < rows; row0 += 128) {
        int cnt[2] = {0, 0}, slo[2] = {0, 0};
#pragma unroll
        for (int q = 0; q < 2; ++q) {
            const int row = row0 + 2 * lane + q;
            if (row < rows) {
                const int pi = (int)(((float)row + 0.5f) * inv_nr);
                const int jr = row - pi * bx.nr;
                const float ux = fmaf(-(float)pi, step, ux0), uy = fmaf(-(float)jr, step, uy0);
                const float h2 = p.c2k - (ux * ux + uy * uy);
                if (h2 > 0.0f) {
                    const float hv = __builtin_amdgcn_sqrtf(h2) * inv_step + 1.0e-3f;
                    const int klo = max(bx.klo, (int)ceilf(fz - hv));
                    const int khi = min(bx.khi, (int)floorf(fz + hv));
                    if (khi >= klo) {       // 4-voxel slots from the chord's first voxel, kept inside the row
                        cnt[q] = (khi - klo + 4) >> 2;
                        slo[q] = ALIGNED ? min(klo, gs.D - 4 * cnt[q]) : klo;
                    }
                }
            }
        }
        const int mine = cnt[0] + cnt[1];
        const int incl = wave_inclusive_scan(mine);
        const int total = bcast(incl, 63);
        const int excl = incl - mine;
        if (mine > 0) marks[excl] = (unsigned char)(lane + 1);
        const int word = excl | (cnt[0] << 11), starts = slo[0] | (slo[1] << 16);
        lds_sync();
        int carry = 0;
        for (int base = 0; base < total; base += 64) {
            const int sidx = base + lane;
            int v = sidx < total ? (int)marks[sidx] : 0;
            v = max(wave_inclusive_max(v), carry);
            carry = bcast(v, 63);
            const int owner = v - 1;
            const int w = __builtin_amdgcn_ds_bpermute(owner << 2, word);
            const int st = __builtin_amdgcn_ds_bpermute(owner << 2, starts);
            if (sidx < total) {
                const int o = sidx - (w & 0x7ff);
                const int c0 = w >> 11;
                const int q = o >= c0 ? 1 : 0;
                const int k4 = q ? (st >> 16) + 4 * (o - c0) : (st & 0xffff) + 4 * o;
                const int row = row0 + 2 * owner + q;
                const int pi = (int)(((float)row + 0.5f) * inv_nr);
                const int jr = row - pi * bx.nr;
                body(off0 + ((unsigned)pi * D + (unsigned)jr) * D, k4,
                     fmaf(-(float)pi, step, ux0), fmaf(-(float)jr, step, uy0));
            }
        }
        lds_sync();
        if (mine > 0) marks[excl] = 0;
        lds_sync();
    }
}

// One atom against kChanGroup channels (Gq[q]: the volume of the q-th of them).
//   (sx, sy, sz) += sum_q cq sum G_q f_q u   (u in units of rmax/sqrt(k)),  sv[q] += sum G_q rho_q
template <bool ALIGNED, bool WANT_W, typename GT>
__device__ inline void reduce_group(const BwdParams &p, const GT *const (&Gq)[kChanGroup],
                                    const float4 &a, float rmax, const Box &bx, float ox, float oy,
                                    float oz, unsigned char *marks, const GroupCoef &gc, float &sx,
                                    float &sy, float &sz, float (&sv)[kChanGroup])
{
    const float s = p.sk * __builtin_amdgcn_rcpf(rmax), step = p.gs.res * s;
    const float azs = (a.z - oz) * s;
    for_each_slot<ALIGNED>(p, a, rmax, bx, ox, oy, oz, marks,
                  [&](unsigned row_off, int k4, float ux, float uy) {
        SlotData d[kChanGroup];
#pragma unroll
        for (int q = 0; q < kChanGroup; ++q)
            if (gc.live[q]) load_slot<ALIGNED, false>(p, Gq[q], row_off, k4, ux, uy, d[q]);
        const float b2 = ux * ux + uy * uy;
        const float uz0 = fmaf(-(float)k4, step, azs);
        float fsum = 0.0f;
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const float uz = uz0 - (float)u * step;
            const float x2m = fmaf(uz, uz, b2);
            // (One square root and one reciprocal square root per voxel, shared by the channels
            // through constants per channel, executes fewer instructions but needs 108 registers
            // instead of 90 -- four wavefronts per SIMD instead of five -- and measured 1.016 ms
            // against 0.99 ms.)
            float F = 0.0f;
#pragma unroll
            for (int q = 0; q < kChanGroup; ++q) {
                if (!gc.live[q]) continue;
                const float x2 = x2m * gc.ratio2[q];
                const float e = __builtin_amdgcn_exp2f(-x2);
                const float rs = __builtin_amdgcn_rsqf(x2);
                const float ft = __builtin_amdgcn_fmed3f(fmaf(p.hAck, rs, -p.hA), 0.0f, 1.0f);
                const float f = x2 <= p.g2k ? e : ft;       // -f/4
                F = fmaf(gc.cq[q], d[q].gv[u] * f, F);
                if (WANT_W) {
                    const float tl = __builtin_amdgcn_fmed3f(fmaf(-(x2 * rs), p.sAk, p.cA), 0.0f, 1.0f);     // sqrt(A) (c - x), clamped to [0, 1]
                    const float rho = x2 <= p.g2k ? e : tl * tl;
                    sv[q] = fmaf(d[q].gv[u], rho, sv[q]);
                }
            }
            fsum += F;
            sz = fmaf(F, uz, sz);
        }
        sx = fmaf(fsum, ux, sx);
        sy = fmaf(fsum, uy, sy);
    });
}

template <bool VECTOR, bool ALIGNED, typename GT>
__global__ __launch_bounds__(256) void backward_kernel(BwdParams p)
{
    const GridSpec &gs = p.gs;
    // The kernel arguments the first loads need are fetched together (they are inputs of an
    // asm statement whose result, zero, enters the example index) instead of in several
    // dependent trips to the scalar cache.
    unsigned zero;
    asm("s_mov_b32 %0, 0"
        : "=s"(zero)
        : "s"((unsigned long long)p.meta), "s"((unsigned long long)p.rec),
          "s"((unsigned long long)p.idx), "s"((unsigned long long)p.gcen),
          "s"((unsigned long long)p.rot), "s"(p.N), "s"(p.T), "s"(p.share), "s"(p.units),
          "s"(p.wgs_per_example), "s"(p.wg_magic));
    // Workgroup ids go round the 8 XCDs (id % 8), each with its own L2.  XCD k takes the k-th
    // eighth of the (example, record) list, so the gradient volume of an example -- and the
    // lines of it that neighbouring records share -- is read through one L2 only.
    if (p.expect_tag != 0u && *p.tag != p.expect_tag) return;      // not the tables this call expects
    const unsigned lin = blockIdx.x + zero;
    const unsigned v = (lin & 7u) * p.share + (lin >> 3);
    if (v >= p.units || (lin >> 3) >= p.share) return;
    const unsigned bu = p.wg_magic == 0ull ? v : (unsigned)__umul64hi((unsigned long long)v, p.wg_magic);
    const int b = (int)bu, slot = (int)((v - bu * p.wgs_per_example) * 4u + (threadIdx.x >> 6));
    const int lane = (int)(threadIdx.x & 63u);
    const int N = p.N, T = p.T, D = gs.D;

    __shared__ __attribute__((aligned(16))) unsigned char s_marks[4][kSlotCap];
    unsigned char *marks = s_marks[threadIdx.x >> 6];
    static_assert(kSlotCap == 64 * 16, "one 16-byte store per lane clears the marks");
    reinterpret_cast<int4 *>(marks)[lane] = make_int4(0, 0, 0, 0);
    lds_sync();
    // Everything the wavefront needs first is requested in one go (one trip to memory, not
    // four in a row): the group table's last entry, the record and its atom index (slot
    // clamped into the array; whether the slot is live is decided afterwards), the grid
    // centre and the rotation.
    const int cslot = min(slot, N - 1);
    const unsigned char atom_alive = p.alive[(size_t)b * N + cslot];    // of ATOM number `slot`, see below
    const int4 last = p.meta[(size_t)b * T + (VECTOR ? 0 : T - 1)];
    const float4 a = p.rec[(size_t)b * N + cslot];
    const int ai = p.idx[(size_t)b * N + cslot];
    const int t_rec = VECTOR ? 0 : p.rchan[(size_t)b * N + cslot];
    const float4 gc = *reinterpret_cast<const float4 *>(p.gcen + 4 * b);
    const float *Rp = p.rot + b * 12;
    const float4 Ra = *reinterpret_cast<const float4 *>(Rp);
    const float4 Rb = *reinterpret_cast<const float4 *>(Rp + 4);
    const float Rc = Rp[8];
    asm volatile("" ::"s"(last.x), "s"(last.z), "s"(gc.x), "s"(gc.y), "s"(gc.z), "s"(Ra.x), "s"(Ra.y),
                 "s"(Ra.z), "s"(Ra.w), "s"(Rb.x), "s"(Rb.y), "s"(Rb.z), "s"(Rb.w), "s"(Rc));
    // Every output element is written by someone: the wavefront of record slot s also looks
    // after ATOM s -- if that atom has no live record (culled, past natoms, type out of range)
    // nobody else writes its gradient, so its zeros are stored here.
    if (slot < N && atom_alive == 0) {
        const size_t atom = (size_t)b * N + slot;
        if (p.grad_coords && lane < 3) p.grad_coords[atom * 3 + lane] = 0.0f;
        if (VECTOR && p.grad_weights)
            for (int k = lane; k < T; k += 64) p.grad_weights[atom * T + k] = 0.0f;
    }
    if (slot >= last.x + last.z) return;            // past the last group's slots (per wavefront)
    if (!(a.w > 0.0f)) return;                      // dead record: its atom's zeros are written above, by slot
    const size_t D3 = (size_t)D * D * D;
    const int bs = source_example(p.subgrids, b);          // types and weights are the source example's
    const float ox = gc.x - gs.half;
    const float oy = gc.y - gs.half;
    const float oz = gc.z - gs.half;

    float tx = 0.0f, ty = 0.0f, tz = 0.0f;          // gradient in the transformed frame
    if (!VECTOR) {
        const int t = t_rec;
        const float r = a.w;
        Box bx;
        float sx = 0.0f, sy = 0.0f, sz = 0.0f, sv = 0.0f;
        if (atom_box(gs, r * gs.c, a, ox, oy, oz, bx))
            reduce_channel<ALIGNED, false>(p, reinterpret_cast<const GT *>(p.G) + (size_t)b * T * D3, t, D3, a, r, bx, ox, oy, oz,
                                           marks, sx, sy, sz, sv);
        // -4 (the sums hold -f/4) / r^2 times r/sqrt(k) (they are in scaled units)
        const float inv_r2 = -4.0f * __builtin_amdgcn_rcpf(r * p.sk);
        tx = wave_sum(sx) * inv_r2;
        ty = wave_sum(sy) * inv_r2;
        tz = wave_sum(sz) * inv_r2;
    } else {
        const size_t arow = ((size_t)bs * N + ai) * T;
        // The channels are taken in order of radius (T <= 64: lane l ranks channel l among the
        // others; more channels are taken as they come), so that the spheres of a group are
        // nearly the same size and few voxels of the widest lie outside the others.
        __shared__ unsigned char s_perm[4][64];
        unsigned char *perm = s_perm[threadIdx.x >> 6];
        const bool sorted = T <= 64;
        if (sorted) {
            float mine = lane < T ? p.radii[lane] : 0.0f;
            mine = mine > 0.0f ? mine : 0.0f;       // NaN and negative radii rank as 0: still a permutation
            int rank = 0;
            for (int m = 0; m < T; ++m) {
                const float other = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(mine), m));
                rank += (other < mine || (other == mine && m < lane)) ? 1 : 0;
            }
            if (lane < T) perm[rank] = (unsigned char)lane;
            lds_sync();
        }
        for (int t0 = 0; t0 < T; t0 += kChanGroup) {
            float rq[kChanGroup], wq[kChanGroup];
            int tq[kChanGroup];
            const GT *Gq[kChanGroup];
            GroupCoef gc;
            float rmax = 0.0f;
#pragma unroll
            for (int q = 0; q < kChanGroup; ++q) {
                const int pos = min(t0 + q, T - 1);
                tq[q] = sorted ? min(__builtin_amdgcn_readfirstlane((int)perm[pos]), T - 1) : pos;
                rq[q] = gs.radius_scale * p.radii[tq[q]];
                wq[q] = p.weights[arow + tq[q]];
                Gq[q] = reinterpret_cast<const GT *>(p.G) + ((size_t)b * T + tq[q]) * D3;
                gc.live[q] = t0 + q < T && rq[q] > 0.0f;
                if (gc.live[q]) rmax = fmaxf(rmax, rq[q]);
            }
            float sx = 0.0f, sy = 0.0f, sz = 0.0f, sv[kChanGroup];
#pragma unroll
            for (int q = 0; q < kChanGroup; ++q) {
                const float inv = gc.live[q] ? __builtin_amdgcn_rcpf(rq[q]) : 0.0f;
                const float ratio = rmax * inv;
                gc.ratio2[q] = ratio * ratio;
                gc.cq[q] = -4.0f * (wq[q] * ratio * inv * p.inv_sk);
                sv[q] = 0.0f;
            }
            Box bx;
            if (rmax > 0.0f && atom_box(gs, rmax * gs.c, a, ox, oy, oz, bx))
            {
                if (p.grad_weights)
                    reduce_group<ALIGNED, true>(p, Gq, a, rmax, bx, ox, oy, oz, marks, gc, sx, sy, sz, sv);
                else
                    reduce_group<ALIGNED, false>(p, Gq, a, rmax, bx, ox, oy, oz, marks, gc, sx, sy, sz, sv);
            }
            tx += sx;       // per lane; summed over the wavefront once, after the last group
            ty += sy;
            tz += sz;
            if (p.grad_weights) {
#pragma unroll
                for (int q = 0; q < kChanGroup; ++q) {
                    if (t0 + q >= T) break;
                    const float val = wave_sum(sv[q]);
                    if (lane == 0) p.grad_weights[((size_t)b * N + ai) * T + tq[q]] = val;
                }
            }
        }
    }
    if (VECTOR && p.grad_coords) {
        tx = wave_sum(tx);
        ty = wave_sum(ty);
        tz = wave_sum(tz);
    }
    if (lane == 0 && p.grad_coords) {
        float *o = p.grad_coords + ((size_t)b * N + ai) * 3;
        o[0] = (Ra.x * tx + Ra.w * ty) + Rb.z * tz;         // R^T: column m of R
        o[1] = (Ra.y * tx + Rb.x * ty) + Rb.w * tz;
        o[2] = (Ra.z * tx + Rb.y * ty) + Rc * tz;
    }
}

// out[b][k] = sum over s < sub3 of tmp[b * sub3 + s][k], summed in order of s
__global__ __launch_bounds__(256) void sum_subgrids_kernel(int sub3, size_t per_example,
                                                           const float *tmp, float *out)
{
    const size_t k = (size_t)blockIdx.x * 256u + threadIdx.x;
    if (k >= per_example) return;
    const size_t b = blockIdx.y;
    const float *src = tmp + b * (size_t)sub3 * per_example + k;
    float acc = 0.0f;
    for (int s = 0; s < sub3; ++s) acc += src[(size_t)s * per_example];
    out[b * per_example + k] = acc;
}

}  // namespace

hipError_t launch_sum_subgrids(int subgrid_count, int B_source, size_t per_example,
                               const float *tmp, float *grad, hipStream_t stream)
{
    const dim3 grd((unsigned)((per_example + 255) / 256), B_source), blk(256);
    hipLaunchKernelGGL(sum_subgrids_kernel, grd, blk, 0, stream, subgrid_count, per_example, tmp, grad);
    return hipGetLastError();
}

hipError_t launch_backward(const GridSpec &gs, const Batch &bt, const Workspace &ws,
                           const void *grad_out, bool grad_is_double, float *grad_coords,
                           float *grad_weights, unsigned expect_tag, KernelEvents ev,
                           hipStream_t stream)
{
    BwdParams p;
    p.gs = gs;
    p.rec = ws.rec; p.idx = ws.idx; p.meta = ws.meta; p.rot = ws.rot;
    p.rchan = ws.rchan; p.weights = bt.weights; p.radii = bt.radii; p.gcen = ws.gcen;
    p.alive = ws.alive; p.tag = ws.tag; p.expect_tag = expect_tag;
    p.G = grad_out; p.grad_coords = grad_coords; p.grad_weights = grad_weights;
    p.subgrids = bt.sub.count; p.N = bt.N; p.T = bt.T;
    {
        const double k = 2.8853900817779268;    // 2 / ln 2
        p.sk = (float)std::sqrt(k);
        p.inv_sk = (float)(1.0 / std::sqrt(k));
        p.g2k = (float)((double)gs.g2 * k);
        p.c2k = (float)((double)gs.c * (double)gs.c * k);
        p.hA = (float)(0.5 * (double)gs.A);
        p.hAck = (float)(0.5 * (double)gs.A * (double)gs.c * std::sqrt(k));
        p.sAk = (float)std::sqrt((double)gs.A / k);
        p.cA = (float)((double)gs.c * std::sqrt((double)gs.A));
    }
    const bool aligned = (gs.D % 4 == 0) && (((uintptr_t)grad_out & 15u) == 0);
    p.wgs_per_example = (unsigned)((bt.N + 3) / 4);
    p.units = p.wgs_per_example * (unsigned)bt.B;
    p.share = (p.units + 7u) / 8u;
    p.wg_magic = p.wgs_per_example <= 1u ? 0ull : (~0ull / p.wgs_per_example) + 1ull;
    const dim3 grd(p.share * 8u), blk(256);
#define MG_BWD(V, Al, Gt) \
    hipExtLaunchKernelGGL((backward_kernel<V, Al, Gt>), grd, blk, 0, stream, ev.start, ev.stop, 0, p)
#define MG_BWD_TYPE(Gt)                                      \
    if (bt.vec) {                                        \
        if (aligned) MG_BWD(true, true, Gt);                 \
        else MG_BWD(true, false, Gt);                        \
    } else {                                                 \
        if (aligned) MG_BWD(false, true, Gt);                \
        else MG_BWD(false, false, Gt);                       \
    }
    if (grad_is_double) { MG_BWD_TYPE(double) } else { MG_BWD_TYPE(float) }
#undef MG_BWD_TYPE
#undef MG_BWD
    return hipGetLastError();
}

}  // namespace mg
