/*
 * molgrid_hip.h -- C ABI of the MI355X (gfx950) atom-to-grid library.
 *
 * The calls follow the problem statement of the libmolgrid paper (arXiv
 * 1912.04822): a GridMaker is built from (resolution, dimension, binary,
 * radius_type_indexed, radius_scale, gaussian_radius_multiple) -- GridMaker
 * constructor listing -- and its forward call turns a batch of typed atoms,
 * each example with an optional rotation/translation (Transformations
 * section), into an N x C x L x W x H float grid (GridMaker usage figure);
 * backward turns a gradient on that grid into atomic gradients (GridMaker
 * section).
 *
 * Conventions for every call
 *   - Returns MG_OK (0) or a negative MG_E* code; nothing throws.  Arguments
 *     are checked on the host before anything is enqueued.
 *   - All array arguments are DEVICE pointers owned by the caller.  The
 *     library allocates nothing: outputs and the workspace are the caller's.
 *   - Work is enqueued on `stream` (a hipStream_t passed as void*, NULL = the
 *     default stream) and the call returns without synchronising.  Calls that
 *     share a workspace must be ordered by the caller (same stream).
 *   - Layouts are dense row-major.  A grid is [B][T][D][D][D] float with the
 *     last (z) index contiguous; grid point (i,j,k) of example b sits at
 *       centers[b] - (D-1)*resolution/2 + resolution*(i,j,k),
 *     D = round(dimension/resolution) + 1 points per side, both ends included.
 *   - natoms[b] (optional) limits example b to its first natoms[b] atoms.
 *     Atoms with a type outside [0,T), a non-positive radius or a non-finite
 *     coordinate contribute nothing and receive zero gradient.
 *   - centers == NULL means the origin, quats == NULL the identity,
 *     translations == NULL zero.  A quaternion is (w,x,y,z) and need not be
 *     normalised; (0,0,0,0) means no rotation.
 *   - Device-side data errors (bad type ids, NaNs) are skipped, not reported.
 */
#ifndef MOLGRID_HIP_H
#define MOLGRID_HIP_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
    MG_OK = 0,
    MG_ENULL = -1,       /* a required pointer is NULL                          */
    MG_ESHAPE = -2,      /* B, N, T < 1, D outside [1, MG_MAX_POINTS], overflow */
    MG_EPARAM = -3,      /* non-finite / non-positive resolution, scale, grm... */
    MG_EWORKSPACE = -4,  /* workspace NULL, misaligned or too small             */
    MG_EHIP = -5,        /* the HIP runtime refused a launch (see mg_last_hip_error) */
    MG_EMODE = -6,       /* call not defined for this GridMaker (e.g. backward in binary mode) */
    MG_EALIGN = -7,      /* a float / int array is not 4-byte (double: 8-byte) aligned */
    MG_ENOMEM = -8       /* the host could not allocate the GridMaker handle     */
};

#define MG_MAX_POINTS 1024      /* largest supported D (points per side) */

typedef struct mg_gridmaker mg_gridmaker;   /* opaque, host-side, immutable after create */

/*
 * GridMaker constructor (constructor listing; defaults there are 0.5, 23.5,
 * 0, 0, 1.0, 1.0).  binary: density is a 0/1 indicator of a voxel lying
 * within radius_scale*radius of an atom instead of the Gaussian-plus-
 * quadratic density.  radius_type_indexed: `radii` is [T], looked up by type
 * id; otherwise it is [B][N], one radius per atom (index types only).
 * gaussian_radius_multiple (grm): the Gaussian runs to grm*r, the quadratic
 * tail reaches zero at r*(1+2grm^2)/(2grm).
 * The handle lives until mg_gridmaker_destroy; *out is set only on MG_OK.
 */
int mg_gridmaker_create(mg_gridmaker **out, float resolution, float dimension,
                        int binary, int radius_type_indexed, float radius_scale,
                        float gaussian_radius_multiple);
void mg_gridmaker_destroy(mg_gridmaker *gm);

/*
 * A GridMaker with a subgrid decomposition (the paper's route to size-
 * extensive models with cubic grids: a larger region is presented as a
 * sequence of cubic subgrids).  The region is a cube of S*D lattice points per
 * side (S = subgrids_per_side, D = round(dimension/resolution)+1, spacing
 * resolution) centred on the example's centre; it is produced as S^3 grids of
 * D points per side, subgrid (sx,sy,sz) holding lattice points
 * [sx*D,(sx+1)*D) x [sy*D,(sy+1)*D) x [sz*D,(sz+1)*D).  Every forward /
 * backward call of such a GridMaker then takes
 *     out, grad_out:  [B][S][S][S][T][D][D][D]   (sx slowest)
 * while all other arrays keep their shapes; gradients are summed over the
 * subgrids; rotation is about the example's centre as before.  A subgrid's
 * centre is, per axis and in float (product, then sum),
 *     centers[b] + ((float)s - (S-1)/2) * ((float)D * resolution).
 * 1 <= S <= MG_MAX_SUBGRIDS and B*S^3 <= 65535 (else MG_ESHAPE); S = 1 is
 * mg_gridmaker_create.  mg_workspace_bytes accounts for S.
 */
#define MG_MAX_SUBGRIDS 16
int mg_gridmaker_create_subgrids(mg_gridmaker **out, float resolution, float dimension,
                                 int subgrids_per_side, int binary, int radius_type_indexed,
                                 float radius_scale, float gaussian_radius_multiple);
int mg_gridmaker_subgrids_per_side(const mg_gridmaker *gm, int *S);

/* D = round(dimension/resolution) + 1. */
int mg_gridmaker_points_per_side(const mg_gridmaker *gm, int *D);

/*
 * Bytes of caller-provided device workspace a forward/backward call with this
 * (B, N, T) needs (transformed, culled, channel-binned atom records).  The
 * workspace must be 32-byte aligned; its contents are scratch.
 */
int mg_workspace_bytes(const mg_gridmaker *gm, int B, int N, int T, size_t *bytes);

/*
 * Transform alone (Transformations section):
 *   out[b][a] = R(quats[b]) (coords[b][a] - centers[b]) + centers[b] + translations[b]
 * coords, out: [B][N][3] float.  The arithmetic is double, in a fixed order,
 * rounded once to float: these are the coordinates forward/backward use.
 */
int mg_transform_forward(int B, int N, const float *coords, const float *centers,
                         const float *quats, const float *translations,
                         float *out, void *stream);

/*
 * The inverse of mg_transform_forward (same arrays, precision and rounding):
 *   out[b][a] = R(quats[b])^T ((coords[b][a] - translations[b]) - centers[b]) + centers[b]
 * The paper shows Transform.forward only; this brings transformed coordinates
 * back to the caller's frame and, with centers = translations = NULL, rotates
 * vectors such as gradients back (R^T v).
 */
int mg_transform_backward(int B, int N, const float *coords, const float *centers,
                          const float *quats, const float *translations,
                          float *out, void *stream);

/*
 * Random augmentation drawn on the device (Transformations section: a random
 * rotation, and a random translation of at most a given distance, per
 * example).  Writes quats [B][4] (w,x,y,z; (1,0,0,0) when random_rotation is
 * 0) and translations [B][3] (zero when max_translation is 0) -- device
 * arrays that the caller then passes to forward / backward, and keeps if the
 * applied transforms are wanted afterwards.
 * The paper fixes no generator or distribution.  Here: Philox4x32-10 with key
 * = seed and counter = (b, draw, block), so example b's transform depends on
 * (seed, draw, b) only (advance `draw` once per batch); a word w becomes
 * u = (w + 0.5) / 2^32; rotation uniform over SO(3) (Shoemake):
 * q = (sqrt(u0) cos 2pi u2, sqrt(1-u0) sin 2pi u1, sqrt(1-u0) cos 2pi u1,
 * sqrt(u0) sin 2pi u2) from block 0; translation t_m = T (2 u_m - 1) per axis
 * from block 1.  Double arithmetic, rounded once to float.
 * max_translation must be finite and >= 0 (else MG_EPARAM).
 */
int mg_draw_transforms(uint64_t seed, uint64_t draw, int B, int random_rotation,
                       float max_translation, float *quats, float *translations,
                       void *stream);

/*
 * Forward, index types (GridMaker section):
 *   out[b][t][p] = sum over atoms a of example b with types[b][a] == t of
 *                  rho(|p - x'_a| / r_a),         r_a = radius_scale * radius
 * or, for a binary GridMaker, 1.0f if any such atom has |p - x'_a| <= r_a
 * (float arithmetic, fixed order) else 0.0f.
 * coords [B][N][3] float; types [B][N] int32; radii [T] or [B][N] float (see
 * create); out [B][T][D][D][D] float, every element written (no need to
 * zero it first).
 */
int mg_forward_index(const mg_gridmaker *gm, int B, int N, int T,
                     const float *coords, const int32_t *types, const float *radii,
                     const int32_t *natoms, const float *centers, const float *quats,
                     const float *translations, float *out,
                     void *workspace, size_t workspace_bytes, void *stream);

/*
 * mg_forward_index for callers that cannot allocate or hand over a workspace
 * (code under HIP graph capture, tight serving loops, harnesses that forbid
 * hipMalloc): the same call and the same kernels, with the workspace in a
 * static device array of MG_STATIC_WORKSPACE_BYTES inside the library (each
 * GPU the library runs on holds its own copy until the process ends).  The
 * call allocates and frees nothing; its first use on a device looks the
 * array's address up (hipGetSymbolAddress), later calls reuse it.  The device
 * of `stream` must be the current device.
 * Returns MG_EWORKSPACE -- before anything is enqueued -- when
 * mg_workspace_bytes(gm, B, N, T) exceeds MG_STATIC_WORKSPACE_BYTES (8 MiB
 * holds B = 50, N = 2040, T = 28 at 48 points per side, 2.6 MB, and B = 16,
 * N = 8000, T = 28 at 96 points, 2.9 MB).
 * All calls on one GPU share that GPU's array: calls that overlap in time
 * (different streams or threads) race; order them.  Nothing in the array has
 * to start at zero: every call writes each table entry before reading it.
 */
#define MG_STATIC_WORKSPACE_BYTES (8u << 20)
int mg_forward_index_static(const mg_gridmaker *gm, int B, int N, int T,
                            const float *coords, const int32_t *types, const float *radii,
                            const int32_t *natoms, const float *centers, const float *quats,
                            const float *translations, float *out, void *stream);

/*
 * Forward, vector types (Atom Typing section: a type may be a vector):
 *   out[b][t][p] = sum_a weights[b][a][t] * rho(|p - x'_a| / (radius_scale * radii[t]))
 * weights [B][N][T] float; radii [T] float, indexed by type id (the GridMaker
 * must have radius_type_indexed set).  Binary GridMaker: 1.0f if any atom
 * with weights[b][a][t] > 0 lies within radius_scale*radii[t].
 */
int mg_forward_vector(const mg_gridmaker *gm, int B, int N, int T,
                      const float *coords, const float *weights, const float *radii,
                      const int32_t *natoms, const float *centers, const float *quats,
                      const float *translations, float *out,
                      void *workspace, size_t workspace_bytes, void *stream);

/*
 * Backward, index types ("computes atomic gradients", GridMaker section):
 * with L = sum(grad_out * out),
 *   grad_coords[b][a] = dL / d coords[b][a]
 *     = R(q_b)^T  sum_p grad_out[b][t_a][p] rho'(d/r_a) (x'_a - p) / (r_a d)
 * grad_out [B][T][D][D][D] float; grad_coords [B][N][3] float, every element
 * written (zero for skipped atoms).  Not defined for a binary GridMaker
 * (MG_EMODE).
 */
int mg_backward_index(const mg_gridmaker *gm, int B, int N, int T,
                      const float *coords, const int32_t *types, const float *radii,
                      const int32_t *natoms, const float *centers, const float *quats,
                      const float *translations, const float *grad_out,
                      float *grad_coords,
                      void *workspace, size_t workspace_bytes, void *stream);

/*
 * Backward, vector types: grad_coords [B][N][3] and grad_weights [B][N][T]
 * (either may be NULL, not both):
 *   grad_coords[b][a]     = R^T sum_t w[b][a][t] sum_p G[b][t][p] rho'(d/r_t)(x'_a - p)/(r_t d)
 *   grad_weights[b][a][t] = sum_p G[b][t][p] rho(d/r_t)
 */
int mg_backward_vector(const mg_gridmaker *gm, int B, int N, int T,
                       const float *coords, const float *weights, const float *radii,
                       const int32_t *natoms, const float *centers, const float *quats,
                       const float *translations, const float *grad_out,
                       float *grad_coords, float *grad_weights,
                       void *workspace, size_t workspace_bytes, void *stream);

/*
 * Tables once, calls many: a training step runs forward and then backward on the
 * same atoms and poses, and both calls begin by building the same tables in the
 * workspace (transformed, culled, channel- and plane-binned records: the
 * transform and culling of the Transformations and GridMaker sections).
 * mg_prepare builds them alone; the *_prepared calls run on them without the
 * prep kernel.  Arguments are as in the ordinary calls; types == NULL in
 * mg_prepare makes the tables of vector types.  The contract is the caller's:
 * the same GridMaker, B, N, T, the same workspace, and nothing else enqueued on
 * that workspace in between (every ordinary forward / backward call rebuilds
 * it); the input arrays must be the ones prepared (weights and radii are read
 * again by the calls that take them).  As a guard, the tables carry a tag
 * of (B, N, T, D, subgrids, kind of types, binary, radius_type_indexed) and the
 * kernels of a *_prepared call whose tag differs return at once and write
 * nothing -- a mismatch leaves the output untouched rather than reading tables
 * of another shape.  Results are those of the ordinary calls, bit for bit.
 */
int mg_prepare(const mg_gridmaker *gm, int B, int N, int T,
               const float *coords, const int32_t *types, const float *radii,
               const int32_t *natoms, const float *centers, const float *quats,
               const float *translations,
               void *workspace, size_t workspace_bytes, void *stream);
int mg_forward_index_prepared(const mg_gridmaker *gm, int B, int N, int T, float *out,
                              void *workspace, size_t workspace_bytes, void *stream);
int mg_forward_vector_prepared(const mg_gridmaker *gm, int B, int N, int T,
                               const float *weights, const float *radii, float *out,
                               void *workspace, size_t workspace_bytes, void *stream);
int mg_backward_index_prepared(const mg_gridmaker *gm, int B, int N, int T,
                               const float *grad_out, float *grad_coords,
                               void *workspace, size_t workspace_bytes, void *stream);
int mg_backward_vector_prepared(const mg_gridmaker *gm, int B, int N, int T,
                                const float *weights, const float *radii, const float *grad_out,
                                float *grad_coords, float *grad_weights,
                                void *workspace, size_t workspace_bytes, void *stream);

/*
 * The same four calls with the grid held in doubles (the paper's grids come
 * in float and double flavours, e.g. a 5-dimensional double grid on the
 * device): out / grad_out are [B][T][D][D][D] double (8-byte aligned); all
 * other arrays, the arithmetic and the results' accuracy are as above (the
 * path computes in float; a double grid holds the same values widened, and
 * a double gradient is narrowed to float as it is read).
 */
int mg_forward_index_f64(const mg_gridmaker *gm, int B, int N, int T,
                         const float *coords, const int32_t *types, const float *radii,
                         const int32_t *natoms, const float *centers, const float *quats,
                         const float *translations, double *out,
                         void *workspace, size_t workspace_bytes, void *stream);
int mg_forward_vector_f64(const mg_gridmaker *gm, int B, int N, int T,
                          const float *coords, const float *weights, const float *radii,
                          const int32_t *natoms, const float *centers, const float *quats,
                          const float *translations, double *out,
                          void *workspace, size_t workspace_bytes, void *stream);
int mg_backward_index_f64(const mg_gridmaker *gm, int B, int N, int T,
                          const float *coords, const int32_t *types, const float *radii,
                          const int32_t *natoms, const float *centers, const float *quats,
                          const float *translations, const double *grad_out,
                          float *grad_coords,
                          void *workspace, size_t workspace_bytes, void *stream);
int mg_backward_vector_f64(const mg_gridmaker *gm, int B, int N, int T,
                           const float *coords, const float *weights, const float *radii,
                           const int32_t *natoms, const float *centers, const float *quats,
                           const float *translations, const double *grad_out,
                           float *grad_coords, float *grad_weights,
                           void *workspace, size_t workspace_bytes, void *stream);

/* Text for an MG_* code (static storage). */
const char *mg_strerror(int code);

/* hipError_t (as int) of the last launch this thread's call refused, 0 if none. */
int mg_last_hip_error(void);

/*
 * Launch knobs, for measurement (results do not depend on them beyond the
 * order of float additions).  Process-wide, each read once per call; setting
 * one while another thread is inside a call affects that call or the next.
 *   "tile_floats"     0, 512, 1024, 2048 or 4096 (default 0 = chosen per call
 *                     from the shapes: 1024 or 2048 for index types, 2048 for
 *                     vector types): consecutive output floats of a channel
 *                     one forward workgroup produces (512: vector types only,
 *                     4096: index types only; otherwise the nearest supported)
 *   "waves_per_tile"  0, 1, 2 or 4 (default 0 = chosen per call: 1 for index
 *                     types, 4 for vector types, whose workgroup produces the
 *                     tiles of four channels): wavefronts in that workgroup
 *                     (never more than tile_floats / 512; 4096-float tiles
 *                     take at least 2)
 *   "xcd_run"         0 or a power of two (default 0): runs of this many
 *                     consecutive tiles go to one XCD
 *   "keep_alive"      0, 1, 64, 128, 256, 512 or 1024 (default 1 = 256): every forward
 *                     wavefront (index types, float grid) also reads that many
 *                     bytes of the workspace tables so that they stay cached while
 *                     the grid is streamed out
 *   "keep_alive_stride" 1, 2, 4 or 8 (default 1): only one wavefront in that many
 *                     does the keep-alive read
 *   "single_launch"   0 or 1 (default 1): index types into a float grid with at most
 *                     256 atoms per example and 2048 in the batch run as ONE kernel
 *                     launch (every tile's wavefront transforms, culls and filters the
 *                     example's atoms itself; no prep kernel, the workspace is not
 *                     touched); 0 = always the prep kernel and its tables.  Binary
 *                     grids are the same to the bit either way, real ones to rounding
 *   "tile_order"      0 or 1 (default 0): 0 = all tiles of a channel, then the
 *                     next channel; 1 = tile k of every channel, then tile k+1
 *   "lds_floor"       -1..65536 (default -1 = chosen per call: 6144 for 4 KB
 *                     tiles of index types, else none): least LDS bytes a forward
 *                     workgroup requests; caps how many are resident on a CU
 * Returns MG_EPARAM for an unknown key or a value outside the ranges above.
 * No knob of the library as built by default can change a result beyond that
 * rounding.  (A measurement build, compiled with -DMG_TIMING_AIDS, also knows
 * "debug" 0..3 -- 1 = no density evaluation, 2 = no atoms, 3 = stores only --
 * and "prep_stop" 0..6 -- end the prep kernel after that stage and skip the
 * main kernel; both leave the output wrong and exist to time parts of a call.)
 */
int mg_set_option(const char *key, int value);

/*
 * Measurement hook: the next forward or backward call made by this thread has
 * `start` stamped when its main kernel (the forward gather / the backward
 * reduction; not the prep kernel) begins and `stop` when it ends.  Both are
 * hipEvent_t handles created by the caller with timing enabled; the hook is
 * cleared by the call that launches.  Pass NULL, NULL to clear it.
 */
int mg_time_next_kernel(void *start_event, void *stop_event);

#ifdef __cplusplus
}
#endif
#endif /* MOLGRID_HIP_H */
