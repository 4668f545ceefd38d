/*
 * molgrid_oracle.c -- TEST INFRASTRUCTURE, NOT PRODUCT CODE.
 *
 * A plain, slow, CPU-only statement of what the atom-to-grid path computes,
 * written from the libmolgrid paper (arXiv 1912.04822): the GridMaker section
 * (density: Gaussian out to grm*r, quadratic decay reaching zero at
 * r*(1+2*grm^2)/(2*grm); binary indicator mode; radius array indexed by type
 * id; radius pre-multiplier; backward = atomic gradients), the GridMaker
 * constructor listing (defaults), the GridMaker usage figure caption (layout
 * N x C x L x W x H) and the Transformations section (rotation by a
 * quaternion about an origin, then a Cartesian translation).
 *
 * Only tests, the smoke check and the CPU-baseline leg of the benchmark may
 * call this file.  It shares no code, header, table or helper with the HIP
 * library and is never a fallback for it.
 *
 * Everything floating-point is double, with two stated exceptions, both
 * because a 0/1 or a stored coordinate is decided there:
 *   - a transformed coordinate is produced in double by one fixed sequence of
 *     operations and then rounded ONCE to float (the library's coordinate
 *     type is a float 3-vector, Transformations section);
 *   - the binary-mode predicate d^2 <= r^2 is evaluated in float with one
 *     fixed operation order and no fused multiply-add.
 * Compile with -ffp-contract=off so the compiler cannot fuse anything.
 *
 * Pins (tests/test_oracle_*.py): peak value 1 at d=0, value and slope
 * continuity at the join, zero value and slope at the cutoff, the closed-form
 * volume integral (erf + polynomial), lattice sum versus quadrature, box
 * variant == brute force bitwise, rotation against scipy's Rotation, 90-degree
 * rotation equivariance, one-hot vector types == index types, ball lattice
 * counts for binary mode (and exact-distance lattice shells for its knife
 * edges), backward against central finite differences and the
 * translational-invariance identity, the Philox known answers, Haar and
 * uniform-box statistics of the drawn transforms, inverse(forward) = identity.
 * Nothing here is "parity unpinned"
 * except agreement with the original libmolgrid binaries, which do not exist
 * in this build (stated in the design notes).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

/* ------------------------------------------------------------------------ */
/* Density (GridMaker section).  x = d / r, g = gaussian_radius_multiple.    */
/* ------------------------------------------------------------------------ */

/* Where the quadratic tail reaches zero, in units of r. */
double orc_cutoff(double g) { return (1.0 + 2.0 * g * g) / (2.0 * g); }

/*
 * The paper fixes: peak-normalised Gaussian for x <= g, a quadratic for
 * g < x < c that "decays to 0" at c = (1+2g^2)/(2g).  A quadratic that lands
 * on zero smoothly is A (x-c)^2.  Joining exp(-a x^2) to it with equal value
 * and slope at x = g gives c = g + 1/(a g); equating with the paper's c
 * forces a = 2 and A = exp(-2 g^2) / (c-g)^2 = 4 g^2 exp(-2 g^2).
 */
double orc_density(double x, double g)
{
    const double c = orc_cutoff(g);
    if (x <= g) return exp(-2.0 * x * x);
    if (x >= c) return 0.0;
    const double A = 4.0 * g * g * exp(-2.0 * g * g);
    return A * (x - c) * (x - c);
}

/* d rho / d x */
double orc_density_deriv(double x, double g)
{
    const double c = orc_cutoff(g);
    if (x <= g) return -4.0 * x * exp(-2.0 * x * x);
    if (x >= c) return 0.0;
    const double A = 4.0 * g * g * exp(-2.0 * g * g);
    return 2.0 * A * (x - c);
}

/* ------------------------------------------------------------------------ */
/* Transform (Transformations section): x' = R(q) (x - c) + c + t.          */
/* q = (w, x, y, z); (1,0,0,0) is the identity, as in the constructor        */
/* listing.  q is normalised by dividing by |q|^2 inside the matrix.         */
/* ------------------------------------------------------------------------ */

void orc_quat_to_matrix(const float *q, double *R)
{
    const double w = q[0], x = q[1], y = q[2], z = q[3];
    const double n = ((w * w + x * x) + y * y) + z * z;
    if (!(n > 0.0) || !isfinite(n)) {          /* no rotation given */
        R[0] = 1; R[1] = 0; R[2] = 0;
        R[3] = 0; R[4] = 1; R[5] = 0;
        R[6] = 0; R[7] = 0; R[8] = 1;
        return;
    }
    const double s = 2.0 / n;
    const double xs = x * s, ys = y * s, zs = z * s;
    const double wx = w * xs, wy = w * ys, wz = w * zs;
    const double xx = x * xs, xy = x * ys, xz = x * zs;
    const double yy = y * ys, yz = y * zs, zz = z * zs;
    R[0] = 1.0 - (yy + zz); R[1] = xy - wz;         R[2] = xz + wy;
    R[3] = xy + wz;         R[4] = 1.0 - (xx + zz); R[5] = yz - wx;
    R[6] = xz - wy;         R[7] = yz + wx;         R[8] = 1.0 - (xx + yy);
}

/* One atom, double in, double out (not yet rounded). */
static void transform_point(const double *R, const double *c, const double *t,
                            const float *p, double *o)
{
    const double u0 = (double)p[0] - c[0];
    const double u1 = (double)p[1] - c[1];
    const double u2 = (double)p[2] - c[2];
    o[0] = (((R[0] * u0 + R[1] * u1) + R[2] * u2) + c[0]) + t[0];
    o[1] = (((R[3] * u0 + R[4] * u1) + R[5] * u2) + c[1]) + t[1];
    o[2] = (((R[6] * u0 + R[7] * u1) + R[8] * u2) + c[2]) + t[2];
}

/* Per-example transform parameters; NULL arrays mean origin / identity / 0. */
typedef struct {
    double R[9], c[3], t[3];
} xform;

static void load_xform(xform *X, int b, const float *centers, const float *quats,
                       const float *translations)
{
    static const float ident[4] = {1.f, 0.f, 0.f, 0.f};
    orc_quat_to_matrix(quats ? quats + 4 * (size_t)b : ident, X->R);
    for (int k = 0; k < 3; ++k) {
        X->c[k] = centers ? (double)centers[3 * (size_t)b + k] : 0.0;
        X->t[k] = translations ? (double)translations[3 * (size_t)b + k] : 0.0;
    }
}

/*
 * Transform a batch.  out32 (float, rounded once) and out64 (double, not
 * rounded) are each optional.  Returns 0.
 */
int orc_transform(int B, int N, const float *coords, const float *centers,
                  const float *quats, const float *translations,
                  float *out32, double *out64)
{
    for (int b = 0; b < B; ++b) {
        xform X;
        load_xform(&X, b, centers, quats, translations);
        for (int a = 0; a < N; ++a) {
            const size_t k = ((size_t)b * N + a) * 3;
            double o[3];
            transform_point(X.R, X.c, X.t, coords + k, o);
            for (int m = 0; m < 3; ++m) {
                if (out32) out32[k + m] = (float)o[m];
                if (out64) out64[k + m] = o[m];
            }
        }
    }
    return 0;
}

/*
 * Inverse of the transform above:  x = R^T ((x' - t) - c) + c, double, fixed
 * order, rounded once for out32.  (The paper shows Transform.forward only;
 * the inverse is what brings transformed coordinates, and with c = t = 0
 * gradient vectors, back to the caller's frame.)
 */
int orc_transform_inverse(int B, int N, const float *coords, const float *centers,
                          const float *quats, const float *translations,
                          float *out32, double *out64)
{
    for (int b = 0; b < B; ++b) {
        xform X;
        load_xform(&X, b, centers, quats, translations);
        for (int a = 0; a < N; ++a) {
            const size_t k = ((size_t)b * N + a) * 3;
            double u[3], o[3];
            for (int m = 0; m < 3; ++m) u[m] = ((double)coords[k + m] - X.t[m]) - X.c[m];
            for (int m = 0; m < 3; ++m)
                o[m] = ((X.R[0 + m] * u[0] + X.R[3 + m] * u[1]) + X.R[6 + m] * u[2]) + X.c[m];
            for (int m = 0; m < 3; ++m) {
                if (out32) out32[k + m] = (float)o[m];
                if (out64) out64[k + m] = o[m];
            }
        }
    }
    return 0;
}

/* ------------------------------------------------------------------------ */
/* Random augmentation (Transformations section: a random rotation and a     */
/* random translation of at most a given distance per example, drawn inside  */
/* GridMaker.forward or by a Transform).  The paper names no generator and   */
/* no distribution; the reading taken here:                                  */
/*   - generator: Philox4x32-10 (Salmon, Moraes, Dror, Shaw, "Parallel       */
/*     random numbers: as easy as 1, 2, 3", SC'11), key = the 64-bit seed    */
/*     (low word, high word), counter = (example index b, low and high word  */
/*     of a 64-bit draw number the caller advances per batch, block), block  */
/*     0 for the rotation and 1 for the translation;                         */
/*   - a 32-bit word w becomes the uniform u = (w + 0.5) / 2^32 in (0, 1);   */
/*   - rotation: uniform over SO(3) by Shoemake's construction ("Uniform     */
/*     random rotations", Graphics Gems III, 1992) from the first three      */
/*     words of block 0:  s1 = sqrt(1-u0), s2 = sqrt(u0), a1 = 2 pi u1,      */
/*     a2 = 2 pi u2,  q = (w,x,y,z) = (s2 cos a2, s1 sin a1, s1 cos a1,      */
/*     s2 sin a2);                                                           */
/*   - translation: each axis uniform in [-T, T], t_m = T (2 u_m - 1) from   */
/*     the first three words of block 1.                                     */
/* Everything is double and rounded once to float.                           */
/* ------------------------------------------------------------------------ */

static void mulhilo32(uint32_t a, uint32_t b, uint32_t *hi, uint32_t *lo)
{
    const uint64_t p = (uint64_t)a * (uint64_t)b;
    *hi = (uint32_t)(p >> 32);
    *lo = (uint32_t)p;
}

/* Ten rounds of the Philox-4x32 bijection; the key is bumped by the Weyl
   constants (golden ratio, sqrt(3)-1) between rounds. */
void orc_philox4x32_10(const uint32_t *ctr, const uint32_t *key, uint32_t *out)
{
    uint32_t c0 = ctr[0], c1 = ctr[1], c2 = ctr[2], c3 = ctr[3];
    uint32_t k0 = key[0], k1 = key[1];
    for (int round = 0; round < 10; ++round) {
        uint32_t hi0, lo0, hi1, lo1;
        mulhilo32(0xD2511F53u, c0, &hi0, &lo0);
        mulhilo32(0xCD9E8D57u, c2, &hi1, &lo1);
        const uint32_t n0 = hi1 ^ c1 ^ k0, n1 = lo1, n2 = hi0 ^ c3 ^ k1, n3 = lo0;
        c0 = n0; c1 = n1; c2 = n2; c3 = n3;
        k0 += 0x9E3779B9u;
        k1 += 0xBB67AE85u;
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

static double word_to_uniform(uint32_t w) { return ((double)w + 0.5) * (1.0 / 4294967296.0); }

/*
 * Per-example random transforms.  quats [B][4] (w,x,y,z), translations [B][3].
 * random_rotation == 0 gives the identity quaternion (1,0,0,0);
 * max_translation == 0 gives zero translations.  Example b's draw depends on
 * (seed, draw, b) only.
 */
int orc_draw_transforms(uint64_t seed, uint64_t draw, int B, int random_rotation,
                        double max_translation, float *quats, float *translations)
{
    const uint32_t key[2] = {(uint32_t)seed, (uint32_t)(seed >> 32)};
    const double two_pi = 6.283185307179586476925286766559;
    for (int b = 0; b < B; ++b) {
        uint32_t ctr[4] = {(uint32_t)b, (uint32_t)draw, (uint32_t)(draw >> 32), 0u}, w[4];
        float *q = quats + 4 * (size_t)b, *t = translations + 3 * (size_t)b;
        if (random_rotation) {
            orc_philox4x32_10(ctr, key, w);
            const double u0 = word_to_uniform(w[0]);
            const double a1 = two_pi * word_to_uniform(w[1]);
            const double a2 = two_pi * word_to_uniform(w[2]);
            const double s1 = sqrt(1.0 - u0), s2 = sqrt(u0);
            q[0] = (float)(s2 * cos(a2));
            q[1] = (float)(s1 * sin(a1));
            q[2] = (float)(s1 * cos(a1));
            q[3] = (float)(s2 * sin(a2));
        } else {
            q[0] = 1.f; q[1] = 0.f; q[2] = 0.f; q[3] = 0.f;
        }
        if (max_translation != 0.0) {
            ctr[3] = 1u;
            orc_philox4x32_10(ctr, key, w);
            for (int m = 0; m < 3; ++m)
                t[m] = (float)(max_translation * (2.0 * word_to_uniform(w[m]) - 1.0));
        } else {
            t[0] = 0.f; t[1] = 0.f; t[2] = 0.f;
        }
    }
    return 0;
}

/* ------------------------------------------------------------------------ */
/* Grid geometry.  D points per side, both ends included; point i along an   */
/* axis sits at  center - (D-1)*res/2 + i*res.  Layout [b][t][ix][iy][iz],   */
/* iz contiguous (usage figure caption: N x C x L x W x H).                  */
/* ------------------------------------------------------------------------ */

int orc_points_per_side(double resolution, double dimension)
{
    return (int)floor(dimension / resolution + 0.5) + 1;
}

typedef struct {
    int B, N, T, D;
    double res, half;           /* half = (D-1)*res/2 */
    double g, cut_mult;         /* grm and c(grm) */
    double radius_scale;
    int radius_type_indexed;    /* 1: radii[T] looked up by type; 0: radii[B,N] per atom */
    int coords_as_float;        /* 1: use the float-rounded transformed coordinate */
} setup;

static void make_setup(setup *S, int B, int N, int T, double res, double dimension,
                       double g, double radius_scale, int radius_type_indexed,
                       int coords_as_float)
{
    S->B = B; S->N = N; S->T = T;
    S->D = orc_points_per_side(res, dimension);
    S->res = res;
    S->half = 0.5 * (S->D - 1) * res;
    S->g = g;
    S->cut_mult = orc_cutoff(g);
    S->radius_scale = radius_scale;
    S->radius_type_indexed = radius_type_indexed;
    S->coords_as_float = coords_as_float;
}

static int atom_count(const setup *S, const int32_t *natoms, int b)
{
    if (!natoms) return S->N;
    int n = natoms[b];
    if (n < 0) n = 0;
    if (n > S->N) n = S->N;
    return n;
}

/* Transformed position of atom (b,a) as the oracle uses it downstream. */
static int atom_position(const setup *S, const xform *X, const float *coords,
                         int b, int a, double *pos)
{
    transform_point(X->R, X->c, X->t, coords + ((size_t)b * S->N + a) * 3, pos);
    for (int m = 0; m < 3; ++m) {
        if (S->coords_as_float) pos[m] = (double)(float)pos[m];
        if (!isfinite(pos[m])) return 0;      /* non-finite atoms are skipped */
    }
    return 1;
}

/* Index range of grid points within `reach` of coordinate p along one axis,
 * widened by one point each side (the density itself decides membership). */
static void axis_range(const setup *S, double origin, double p, double reach,
                       int *lo, int *hi)
{
    double l = floor((p - reach - origin) / S->res) - 1.0;
    double h = ceil((p + reach - origin) / S->res) + 1.0;
    if (l < 0.0) l = 0.0;
    if (h > S->D - 1.0) h = S->D - 1.0;
    *lo = (int)l;
    *hi = (int)h;   /* may be < lo: empty */
}

/* Add one atom's density into one channel grid (D^3 doubles). */
static void add_atom_real(const setup *S, const xform *X, double *chan,
                          const double *pos, double r, double weight, int box)
{
    const int D = S->D;
    int lo[3] = {0, 0, 0}, hi[3] = {D - 1, D - 1, D - 1};
    if (box)
        for (int m = 0; m < 3; ++m)
            axis_range(S, X->c[m] - S->half, pos[m], r * S->cut_mult, &lo[m], &hi[m]);
    for (int i = lo[0]; i <= hi[0]; ++i) {
        const double dx = (X->c[0] - S->half + i * S->res) - pos[0];
        for (int j = lo[1]; j <= hi[1]; ++j) {
            const double dy = (X->c[1] - S->half + j * S->res) - pos[1];
            for (int k = lo[2]; k <= hi[2]; ++k) {
                const double dz = (X->c[2] - S->half + k * S->res) - pos[2];
                const double d = sqrt(dx * dx + dy * dy + dz * dz);
                const double v = orc_density(d / r, S->g);
                if (v != 0.0) chan[((size_t)i * D + j) * D + k] += weight * v;
            }
        }
    }
}

static void emit(const double *acc, size_t n, float *out32, double *out64)
{
    for (size_t i = 0; i < n; ++i) {
        if (out32) out32[i] = (float)acc[i];
        if (out64) out64[i] = acc[i];
    }
}

/*
 * Real-valued forward, index types.
 *   out[b,t,p] = sum over atoms a of example b with type t of rho(|p - x'_a| / r_a)
 * box = 0: every atom against every voxel; box = 1: only the voxels of the
 * atom's cutoff cube.  radii is [T] when radius_type_indexed, else [B,N].
 * Atoms with type < 0 or >= T, or non-finite position, are skipped.
 * out32 / out64: [B,T,D,D,D], each optional.  threads <= 0: OpenMP default.
 * Returns the number of threads used (>= 1), or -1 on allocation failure.
 */
int orc_forward_index(int B, int N, int T, double res, double dimension,
                      double g, double radius_scale, int radius_type_indexed,
                      int coords_as_float, int box,
                      const float *coords, const int32_t *types, const float *radii,
                      const int32_t *natoms, const float *centers, const float *quats,
                      const float *translations, float *out32, double *out64,
                      int threads)
{
    setup S;
    make_setup(&S, B, N, T, res, dimension, g, radius_scale, radius_type_indexed,
               coords_as_float);
    const size_t D3 = (size_t)S.D * S.D * S.D, per_ex = D3 * T;
    int used = 1, fail = 0;
#ifdef _OPENMP
    if (threads > 0) omp_set_num_threads(threads);
#pragma omp parallel
    {
#pragma omp single
        used = omp_get_num_threads();
    }
#endif
#pragma omp parallel for schedule(dynamic, 1)
    for (int b = 0; b < B; ++b) {
        double *acc = (double *)calloc(per_ex, sizeof(double));
        if (!acc) { fail = 1; continue; }
        xform X;
        load_xform(&X, b, centers, quats, translations);
        const int n = atom_count(&S, natoms, b);
        for (int a = 0; a < n; ++a) {
            const int t = types[(size_t)b * N + a];
            if (t < 0 || t >= T) continue;
            double pos[3];
            if (!atom_position(&S, &X, coords, b, a, pos)) continue;
            const double rad = radius_type_indexed ? radii[t] : radii[(size_t)b * N + a];
            const double r = radius_scale * rad;
            if (!(r > 0.0)) continue;
            add_atom_real(&S, &X, acc + (size_t)t * D3, pos, r, 1.0, box);
        }
        emit(acc, per_ex, out32 ? out32 + (size_t)b * per_ex : 0,
             out64 ? out64 + (size_t)b * per_ex : 0);
        free(acc);
    }
    return fail ? -1 : used;
}

/*
 * Real-valued forward, vector types: every atom carries weights[T]; channel t
 * uses radius radius_scale * radii[t] (the radius array is indexed by type id).
 *   out[b,t,p] = sum_a w[b,a,t] * rho(|p - x'_a| / r_t)
 */
int orc_forward_vector(int B, int N, int T, double res, double dimension,
                       double g, double radius_scale, int coords_as_float, int box,
                       const float *coords, const float *weights, const float *radii,
                       const int32_t *natoms, const float *centers, const float *quats,
                       const float *translations, float *out32, double *out64,
                       int threads)
{
    setup S;
    make_setup(&S, B, N, T, res, dimension, g, radius_scale, 1, coords_as_float);
    const size_t D3 = (size_t)S.D * S.D * S.D, per_ex = D3 * T;
    int used = 1, fail = 0;
#ifdef _OPENMP
    if (threads > 0) omp_set_num_threads(threads);
#pragma omp parallel
    {
#pragma omp single
        used = omp_get_num_threads();
    }
#endif
#pragma omp parallel for schedule(dynamic, 1)
    for (int b = 0; b < B; ++b) {
        double *acc = (double *)calloc(per_ex, sizeof(double));
        if (!acc) { fail = 1; continue; }
        xform X;
        load_xform(&X, b, centers, quats, translations);
        const int n = atom_count(&S, natoms, b);
        for (int a = 0; a < n; ++a) {
            double pos[3];
            if (!atom_position(&S, &X, coords, b, a, pos)) continue;
            for (int t = 0; t < T; ++t) {
                const double w = weights[((size_t)b * N + a) * T + t];
                const double r = radius_scale * (double)radii[t];
                if (w == 0.0 || !(r > 0.0)) continue;
                add_atom_real(&S, &X, acc + (size_t)t * D3, pos, r, w, box);
            }
        }
        emit(acc, per_ex, out32 ? out32 + (size_t)b * per_ex : 0,
             out64 ? out64 + (size_t)b * per_ex : 0);
        free(acc);
    }
    return fail ? -1 : used;
}

/* ------------------------------------------------------------------------ */
/* Binary mode: voxel = 1 if any atom of the channel lies within r of it.    */
/* The decision is taken in float, in this exact order, each operation       */
/* rounded on its own:                                                       */
/*   half  = (float)(0.5 * (D-1) * (double)res)                              */
/*   o     = c - half                  (float subtract, per axis)            */
/*   gx    = o + (float)i * res        (float multiply, then float add)      */
/*   dx    = gx - ax                   (ax = float transformed coordinate)   */
/*   d2    = (dx*dx + dy*dy) + dz*dz                                         */
/*   r     = radius_scale * radius     (float multiply)                      */
/*   inside iff d2 <= r*r                                                    */
/* ------------------------------------------------------------------------ */

static void mark_atom_binary(const setup *S, const float *o, float res,
                             float *chan, const float *a, float r, int box)
{
    const int D = S->D;
    int lo[3] = {0, 0, 0}, hi[3] = {D - 1, D - 1, D - 1};
    if (box)
        for (int m = 0; m < 3; ++m)
            axis_range(S, (double)o[m], (double)a[m], (double)r, &lo[m], &hi[m]);
    const float r2 = r * r;
    for (int i = lo[0]; i <= hi[0]; ++i) {
        const float gx = o[0] + (float)i * res;
        const float dx = gx - a[0];
        for (int j = lo[1]; j <= hi[1]; ++j) {
            const float gy = o[1] + (float)j * res;
            const float dy = gy - a[1];
            for (int k = lo[2]; k <= hi[2]; ++k) {
                const float gz = o[2] + (float)k * res;
                const float dz = gz - a[2];
                const float d2 = (dx * dx + dy * dy) + dz * dz;
                if (d2 <= r2) chan[((size_t)i * D + j) * D + k] = 1.0f;
            }
        }
    }
}

/*
 * Binary forward.  Index types when `types` is given; otherwise vector types
 * (`weights` given): channel t is set by any atom with w[a,t] > 0 within
 * radius_scale*radii[t] (this build's definition; the paper does not cover
 * binary with vector types).  out: [B,T,D,D,D] float, values 0.0f / 1.0f.
 */
int orc_forward_binary(int B, int N, int T, float res, float dimension,
                       float radius_scale, int radius_type_indexed, int box,
                       const float *coords, const int32_t *types, const float *weights,
                       const float *radii, const int32_t *natoms, const float *centers,
                       const float *quats, const float *translations, float *out,
                       int threads)
{
    setup S;
    make_setup(&S, B, N, T, (double)res, (double)dimension, 1.0, (double)radius_scale,
               radius_type_indexed, 1);
    const size_t D3 = (size_t)S.D * S.D * S.D, per_ex = D3 * T;
    const float halff = (float)(0.5 * (S.D - 1) * (double)res);
    int used = 1;
#ifdef _OPENMP
    if (threads > 0) omp_set_num_threads(threads);
#pragma omp parallel
    {
#pragma omp single
        used = omp_get_num_threads();
    }
#endif
#pragma omp parallel for schedule(dynamic, 1)
    for (int b = 0; b < B; ++b) {
        float *ex = out + (size_t)b * per_ex;
        memset(ex, 0, per_ex * sizeof(float));
        xform X;
        load_xform(&X, b, centers, quats, translations);
        float o[3];
        for (int m = 0; m < 3; ++m) {
            const float cf = centers ? centers[3 * (size_t)b + m] : 0.0f;
            o[m] = cf - halff;
        }
        const int n = atom_count(&S, natoms, b);
        for (int a = 0; a < n; ++a) {
            double pos[3];
            if (!atom_position(&S, &X, coords, b, a, pos)) continue;
            const float af[3] = {(float)pos[0], (float)pos[1], (float)pos[2]};
            if (types) {
                const int t = types[(size_t)b * N + a];
                if (t < 0 || t >= T) continue;
                const float rad = radius_type_indexed ? radii[t] : radii[(size_t)b * N + a];
                const float r = radius_scale * rad;
                if (!(r > 0.0f)) continue;
                mark_atom_binary(&S, o, res, ex + (size_t)t * D3, af, r, box);
            } else {
                for (int t = 0; t < T; ++t) {
                    if (!(weights[((size_t)b * N + a) * T + t] > 0.0f)) continue;
                    const float r = radius_scale * radii[t];
                    if (!(r > 0.0f)) continue;
                    mark_atom_binary(&S, o, res, ex + (size_t)t * D3, af, r, box);
                }
            }
        }
    }
    return used;
}

/*
 * Knife edges of the binary mode: voxels where, for some atom of the channel,
 * the exact (double) squared distance lies within `eps` of r^2, so that the
 * float predicate above is decided by rounding rather than by geometry.  A
 * binary grid computed in another float order could legitimately differ there
 * and nowhere else.  mask: [B,T,D,D,D] bytes, 1 on a knife edge.  Index types
 * when `types` is given, else vector types as in orc_forward_binary.  The atom
 * position is the float-rounded transformed coordinate (what the predicate
 * sees); the grid point and the radius are taken in double.
 * Pin: an atom on a lattice point with r a multiple of the spacing has as its
 * knife edges exactly the lattice points with i^2+j^2+k^2 = (r/res)^2.
 */
int orc_binary_knife_edges(int B, int N, int T, float res, float dimension,
                           float radius_scale, int radius_type_indexed, double eps,
                           const float *coords, const int32_t *types, const float *weights,
                           const float *radii, const int32_t *natoms, const float *centers,
                           const float *quats, const float *translations,
                           unsigned char *mask)
{
    setup S;
    make_setup(&S, B, N, T, (double)res, (double)dimension, 1.0, (double)radius_scale,
               radius_type_indexed, 1);
    const int D = S.D;
    const size_t D3 = (size_t)D * D * D, per_ex = D3 * T;
    for (int b = 0; b < B; ++b) {
        unsigned char *ex = mask + (size_t)b * per_ex;
        memset(ex, 0, per_ex);
        xform X;
        load_xform(&X, b, centers, quats, translations);
        const int n = atom_count(&S, natoms, b);
        for (int a = 0; a < n; ++a) {
            double pos[3];
            if (!atom_position(&S, &X, coords, b, a, pos)) continue;
            const double af[3] = {(double)(float)pos[0], (double)(float)pos[1], (double)(float)pos[2]};
            const int t0 = types ? types[(size_t)b * N + a] : 0;
            const int t1 = types ? t0 + 1 : T;
            if (types && (t0 < 0 || t0 >= T)) continue;
            for (int t = t0; t < t1; ++t) {
                if (!types && !(weights[((size_t)b * N + a) * T + t] > 0.0f)) continue;
                const float rad = (radius_type_indexed || !types) ? radii[t] : radii[(size_t)b * N + a];
                const double r = (double)radius_scale * (double)rad;
                if (!(r > 0.0)) continue;
                int lo[3], hi[3];
                for (int m = 0; m < 3; ++m)
                    axis_range(&S, X.c[m] - S.half, af[m], r + sqrt(eps) + S.res, &lo[m], &hi[m]);
                for (int i = lo[0]; i <= hi[0]; ++i) {
                    const double dx = (X.c[0] - S.half + i * S.res) - af[0];
                    for (int j = lo[1]; j <= hi[1]; ++j) {
                        const double dy = (X.c[1] - S.half + j * S.res) - af[1];
                        for (int k = lo[2]; k <= hi[2]; ++k) {
                            const double dz = (X.c[2] - S.half + k * S.res) - af[2];
                            const double d2 = dx * dx + dy * dy + dz * dz;
                            if (fabs(d2 - r * r) < eps)
                                ex[(size_t)t * D3 + ((size_t)i * D + j) * D + k] = 1;
                        }
                    }
                }
            }
        }
    }
    return 0;
}

/* ------------------------------------------------------------------------ */
/* Backward (GridMaker section: "computes atomic gradients").               */
/* L = sum G * out.  For one atom and one voxel, with u = x'_a - p,          */
/* d = |u|, x = d/r:   d rho / d x'_a = rho'(x) * u / (r d),  0 at d = 0.    */
/* The gradient with respect to the caller's coordinates is R^T times the    */
/* sum (the center and the translation drop out).                            */
/* ------------------------------------------------------------------------ */

/* Sum over one channel of G * d rho/d x' (grad, 3) and G * rho (value). */
static void reduce_atom(const setup *S, const xform *X, const double *chanG64,
                        const float *chanG32, const double *pos, double r, int box,
                        double *grad, double *value)
{
    const int D = S->D;
    int lo[3] = {0, 0, 0}, hi[3] = {D - 1, D - 1, D - 1};
    if (box)
        for (int m = 0; m < 3; ++m)
            axis_range(S, X->c[m] - S->half, pos[m], r * S->cut_mult, &lo[m], &hi[m]);
    double gx = 0, gy = 0, gz = 0, val = 0;
    for (int i = lo[0]; i <= hi[0]; ++i) {
        const double ux = pos[0] - (X->c[0] - S->half + i * S->res);
        for (int j = lo[1]; j <= hi[1]; ++j) {
            const double uy = pos[1] - (X->c[1] - S->half + j * S->res);
            for (int k = lo[2]; k <= hi[2]; ++k) {
                const double uz = pos[2] - (X->c[2] - S->half + k * S->res);
                const size_t v = ((size_t)i * D + j) * D + k;
                const double G = chanG64 ? chanG64[v] : (double)chanG32[v];
                const double d = sqrt(ux * ux + uy * uy + uz * uz);
                val += G * orc_density(d / r, S->g);
                if (d > 0.0) {
                    const double f = G * orc_density_deriv(d / r, S->g) / (r * d);
                    gx += f * ux; gy += f * uy; gz += f * uz;
                }
            }
        }
    }
    grad[0] = gx; grad[1] = gy; grad[2] = gz;
    *value = val;
}

static void rotate_back(const double *R, const double *g, double *o)
{
    o[0] = (R[0] * g[0] + R[3] * g[1]) + R[6] * g[2];
    o[1] = (R[1] * g[0] + R[4] * g[1]) + R[7] * g[2];
    o[2] = (R[2] * g[0] + R[5] * g[1]) + R[8] * g[2];
}

/*
 * Backward, index types.  grad_out is [B,T,D,D,D] (float G32 or double G64,
 * exactly one non-NULL); grad_coords [B,N,3] double, fully overwritten
 * (skipped / padded atoms get 0).
 */
int orc_backward_index(int B, int N, int T, double res, double dimension,
                       double g, double radius_scale, int radius_type_indexed,
                       int coords_as_float, int box,
                       const float *coords, const int32_t *types, const float *radii,
                       const int32_t *natoms, const float *centers, const float *quats,
                       const float *translations, const float *G32, const double *G64,
                       double *grad_coords, int threads)
{
    setup S;
    make_setup(&S, B, N, T, res, dimension, g, radius_scale, radius_type_indexed,
               coords_as_float);
    const size_t D3 = (size_t)S.D * S.D * S.D, per_ex = D3 * T;
    int used = 1;
#ifdef _OPENMP
    if (threads > 0) omp_set_num_threads(threads);
#pragma omp parallel
    {
#pragma omp single
        used = omp_get_num_threads();
    }
#endif
#pragma omp parallel for schedule(dynamic, 1)
    for (int b = 0; b < B; ++b) {
        xform X;
        load_xform(&X, b, centers, quats, translations);
        const int n = atom_count(&S, natoms, b);
        for (int a = 0; a < N; ++a) {
            double *out = grad_coords + ((size_t)b * N + a) * 3;
            out[0] = out[1] = out[2] = 0.0;
            if (a >= n) continue;
            const int t = types[(size_t)b * N + a];
            if (t < 0 || t >= T) continue;
            double pos[3];
            if (!atom_position(&S, &X, coords, b, a, pos)) continue;
            const double rad = radius_type_indexed ? radii[t] : radii[(size_t)b * N + a];
            const double r = radius_scale * rad;
            if (!(r > 0.0)) continue;
            const size_t off = (size_t)b * per_ex + (size_t)t * D3;
            double gp[3], val;
            reduce_atom(&S, &X, G64 ? G64 + off : 0, G32 ? G32 + off : 0, pos, r, box,
                        gp, &val);
            rotate_back(X.R, gp, out);
        }
    }
    return used;
}

/*
 * Backward, vector types.  grad_coords [B,N,3] and grad_weights [B,N,T]
 * (double, each optional, fully overwritten):
 *   dL/dx'_a   = sum_t w[a,t] sum_v G[t,v] rho'(d/r_t) u / (r_t d)
 *   dL/dw[a,t] = sum_v G[t,v] rho(d/r_t)
 * The weight gradient does not depend on w, so it is produced for zero
 * weights too.
 */
int orc_backward_vector(int B, int N, int T, double res, double dimension,
                        double g, double radius_scale, int coords_as_float, int box,
                        const float *coords, const float *weights, const float *radii,
                        const int32_t *natoms, const float *centers, const float *quats,
                        const float *translations, const float *G32, const double *G64,
                        double *grad_coords, double *grad_weights, int threads)
{
    setup S;
    make_setup(&S, B, N, T, res, dimension, g, radius_scale, 1, coords_as_float);
    const size_t D3 = (size_t)S.D * S.D * S.D, per_ex = D3 * T;
    int used = 1;
#ifdef _OPENMP
    if (threads > 0) omp_set_num_threads(threads);
#pragma omp parallel
    {
#pragma omp single
        used = omp_get_num_threads();
    }
#endif
#pragma omp parallel for schedule(dynamic, 1)
    for (int b = 0; b < B; ++b) {
        xform X;
        load_xform(&X, b, centers, quats, translations);
        const int n = atom_count(&S, natoms, b);
        for (int a = 0; a < N; ++a) {
            const size_t ia = (size_t)b * N + a;
            double acc[3] = {0, 0, 0};
            if (grad_weights)
                for (int t = 0; t < T; ++t) grad_weights[ia * T + t] = 0.0;
            double pos[3];
            const int live = a < n && atom_position(&S, &X, coords, b, a, pos);
            if (live) {
                for (int t = 0; t < T; ++t) {
                    const double r = radius_scale * (double)radii[t];
                    if (!(r > 0.0)) continue;
                    const size_t off = (size_t)b * per_ex + (size_t)t * D3;
                    double gp[3], val;
                    reduce_atom(&S, &X, G64 ? G64 + off : 0, G32 ? G32 + off : 0, pos, r,
                                box, gp, &val);
                    const double w = weights[ia * T + t];
                    acc[0] += w * gp[0]; acc[1] += w * gp[1]; acc[2] += w * gp[2];
                    if (grad_weights) grad_weights[ia * T + t] = val;
                }
            }
            if (grad_coords) {
                double o[3];
                rotate_back(X.R, acc, o);
                grad_coords[ia * 3 + 0] = live ? o[0] : 0.0;
                grad_coords[ia * 3 + 1] = live ? o[1] : 0.0;
                grad_coords[ia * 3 + 2] = live ? o[2] : 0.0;
            }
        }
    }
    return used;
}
