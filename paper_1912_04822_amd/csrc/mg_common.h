// Internal declarations shared by the HIP translation units of the library.
// Not part of the C ABI (that is include/molgrid_hip.h).
#pragma once

#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>
#include <stddef.h>
#include <stdint.h>

namespace mg {

// ---------------------------------------------------------------------------
// GridMaker: host-side, immutable.  Constants of the density (GridMaker
// section of the paper): with x = d/r and g = gaussian_radius_multiple,
//   rho(x) = exp(-2 x^2)           x <= g
//          = A (x - c)^2           g < x < c,   c = (1+2g^2)/(2g)
//          = 0                     x >= c
// A = 4 g^2 exp(-2 g^2) makes value and slope continuous at x = g: a Gaussian
// exp(-a x^2) meets a quadratic with a double root at c smoothly only when
// c = g + 1/(a g), which matches the paper's c for a = 2.
// ---------------------------------------------------------------------------
struct GridSpec {
    float res;          // grid spacing
    float half;         // (D-1)*res/2, rounded once from double
    float inv_res;
    int   D;            // points per side
    int   binary;
    int   radius_type_indexed;
    float radius_scale;
    float g2;           // g^2            (Gaussian region is x^2 <= g2)
    float c;            // cutoff multiple (1+2g^2)/(2g)
    float c2;           // c^2
    float A;            // tail coefficient
};

// Subgrid decomposition (the paper's way to stay size-extensive with cubic grids): a cube
// of per_side*D lattice points per side, spacing res, centred on the example's centre, is
// produced as per_side^3 grids of D points per side.  The kernels see count = per_side^3
// "virtual examples" per example: virtual example e reads the atoms and the pose of example
// e / count and owns subgrid e % count = (sx*per_side + sy)*per_side + sz, whose centre is
// centre + ((float)s - mid) * step per axis (float, product then sum).
struct Subgrids {
    int   per_side;     // 1: the plain GridMaker
    int   count;        // per_side^3
    float mid;          // (per_side-1)/2
    float step;         // (float)D * res
};

// the example whose atoms and pose virtual example e reads
__host__ __device__ inline int source_example(int subgrid_count, int e)
{
    return subgrid_count > 1 ? e / subgrid_count : e;
}

// ---------------------------------------------------------------------------
// Workspace layout (device, caller-provided, 32-byte aligned).  A "group" is
// the set of atoms one output channel reads: for index types the atoms of
// example b with type t (group b*T+t), for vector types all atoms of example
// b (group b*T+0).
//   rec   [B][N] float4   transformed atom records {x', y', z', r} (vector
//                         types: r = 1).  The live records of a group sit at
//                         rec[b][first .. first+live), binned by x-plane (bin
//                         k+1 holds floor((x'-origin_x)/res) == k, bins 0 and
//                         D+1 the atoms left / right of the grid) and, inside
//                         a bin, in atom order.  Slots first+live .. first+all
//                         hold w = 0.
//   idx   [B][N] int32    original atom index of each record
//   meta  [B][T] int4     {first, live, all, sorted}; sorted = 0 means the
//                         group was too long to bin: its records are in atom
//                         order, culled ones carry r = 0, and live == all
//   range [B][T][D] int2  for x-plane i: the span [r0, r1) of records, counted from
//                         the example's first record rec[b][0], that can reach
//                         the plane; r0 and r1 do not decrease with i, so planes
//                         i..k are reached by [range[i].x, range[k].y).  The table
//                         is small and every line of it is read by several
//                         forward workgroups: reads that miss L2 while the chip
//                         streams stores cost far more than their bytes
//   rot   [B][12] float   rotation matrix rows (9 used), for the backward pass
//   gcen  [B][4] float    centre of the example's grid (3 used)
//   chan_order [B][T] int32  vector types: the channels in order of radius (ties by index;
//                         as they come beyond kRankCap channels), so that channels taken
//                         together have spheres of nearly the same size
//   alive [B][N] uint8    1 for an atom that has a live record, 0 for one that is culled,
//                         past natoms or of a type outside [0,T): the backward kernels write
//                         the zero gradients of those (the wavefront of record slot s looks
//                         after atom s)
//   rchan [B][N] int32    the channel of each record (index types: the atom's type), so that
//                         the backward kernel has it with the record and not a trip to the
//                         type array later
//   tag   [1] uint32      what the tables were made for (workspace_tag), written last
//   gtmp  [B][N][3] float, wtmp [B][N][T] float: with subgrids only, the
//                         gradients per virtual example before they are summed
// With subgrids B counts virtual examples everywhere above.
// ---------------------------------------------------------------------------
struct Workspace {
    float4 *rec;
    int    *idx;
    int4   *meta;
    int2   *range;
    float  *rot;
    float  *gcen;
    int    *chan_order;
    unsigned char *alive;
    int    *rchan;
    unsigned *tag;
    float  *gtmp;
    float  *wtmp;
};

// B counts virtual examples; subgrid_count > 1 adds the gradient staging
size_t workspace_bytes(const GridSpec &gs, int subgrid_count, int B, int N, int T);
Workspace carve_workspace(const GridSpec &gs, int subgrid_count, void *base, int B, int N, int T);

// B counts virtual examples (see Subgrids); the arrays are indexed by source example.
struct Batch {
    int B, N, T;
    bool vec;                     // vector types (weights) rather than index types
    Subgrids sub;
    const float   *coords;        // [B][N][3]
    const int32_t *types;         // [B][N] or null (vector types)
    const float   *weights;       // [B][N][T] or null (index types)
    const float   *radii;         // [T] or [B][N]
    const int32_t *natoms;        // [B] or null
    const float   *centers;       // [B][3] or null
    const float   *quats;         // [B][4] or null
    const float   *translations;  // [B][3] or null
};

// Geometry of the forward kernel: every wavefront owns one flat tile of
// `tile_floats` consecutive floats of one channel (the last tile of a channel
// may be shorter).
struct ForwardGeometry {
    int tile_floats;    // 1024, 2048 or 4096
    int tiles;          // tiles per channel = ceil(D^3 / tile_floats)
};
ForwardGeometry forward_geometry(int D, int tile_floats);

constexpr int kSortCap = 2048;          // longest group the prep kernel bins by x-plane
constexpr int kRankCap = 256;           // most channels that are put in order of radius

// Timing events for the main kernel of the current call (null: none).  The launchers pass
// them to hipExtLaunchKernelGGL, which stamps them at the start and the end of that very
// kernel.
struct KernelEvents {
    hipEvent_t start, stop;
};

// Timing aids (kernel phases switched off, prep kernel ended after a stage) give wrong grids
// and exist only in a library built with -DMG_TIMING_AIDS (a measurement build); in the
// release library the tests below are compile-time false and their branches vanish.
#ifdef MG_TIMING_AIDS
#define MG_DEBUG_IS(p, n) ((p).debug == (n))
#define MG_STOP_IS(stop, n) ((stop) == (n))
#else
#define MG_DEBUG_IS(p, n) false
#define MG_STOP_IS(stop, n) false
#endif

// Launchers (each enqueues on `stream`, returns the hipError_t of the launch).
hipError_t launch_transform(int B, int N, const float *coords, const float *centers,
                            const float *quats, const float *translations, float *out,
                            bool inverse, hipStream_t stream);
hipError_t launch_draw_transforms(uint64_t seed, uint64_t draw, int B, bool random_rotation,
                                  float max_translation, float *quats, float *translations,
                                  hipStream_t stream);
unsigned workspace_tag(const GridSpec &gs, const Batch &bt);
hipError_t launch_prep(const GridSpec &gs, const Batch &bt, const Workspace &ws, int stop,
                       hipStream_t stream);
// Small problems (index types, float grid): the forward kernel alone, no prep kernel -- every
// tile's wavefront transforms, culls and filters the example's atoms itself.
constexpr int kSmallAtoms = 256;        // most atoms per example
constexpr int kSmallTotal = 2048;       // most atoms in the batch
bool forward_takes_single_launch(const Batch &bt, bool out_is_double);
// expect_tag != 0 (a *_prepared call): the kernel returns at once, writing nothing, unless the
// workspace's tag equals it
hipError_t launch_forward(const GridSpec &gs, const Batch &bt, const Workspace &ws,
                          void *out, bool out_is_double, int tile_floats, int waves_per_tile,
                          int xcd_run, int lds_floor, int debug, int tile_order, int keep_alive,
                          bool single_launch, unsigned expect_tag, KernelEvents ev, hipStream_t stream,
                          int keep_alive_stride = 1);
hipError_t launch_backward(const GridSpec &gs, const Batch &bt, const Workspace &ws,
                           const void *grad_out, bool grad_is_double, float *grad_coords,
                           float *grad_weights, unsigned expect_tag, KernelEvents ev,
                           hipStream_t stream);
// grad[b] = sum over the sub3 virtual examples of b, in order (subgrids only)
hipError_t launch_sum_subgrids(int subgrid_count, int B_source, size_t per_example,
                               const float *tmp, float *grad, hipStream_t stream);

}  // namespace mg
