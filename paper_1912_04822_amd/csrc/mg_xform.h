// The per-example coordinate transform (Transformations section of the paper),
//   x' = R(q)(x - c) + c + t,   q = (w,x,y,z), (1,0,0,0) the identity,
// in the one fixed double-precision sequence every kernel of the library uses (compiled
// with -ffp-contract=off: nothing fuses), rounded once to float:
//   n  = ((w*w + x*x) + y*y) + z*z          s = 2/n   (n == 0: identity)
//   xs = x*s, ys = y*s, zs = z*s
//   R  = [ 1-(y*ys+z*zs)   x*ys-w*zs      x*zs+w*ys   ]
//        [ x*ys+w*zs       1-(x*xs+z*zs)  y*zs-w*xs   ]
//        [ x*zs-w*ys       y*zs+w*xs      1-(x*xs+y*ys) ]
//   x'_m = (((R_m0*u0 + R_m1*u1) + R_m2*u2) + c_m) + t_m,   u = x - c
#pragma once

#include <hip/hip_runtime.h>

namespace mg {

struct Xform {
    double R[9];
    double c[3];
    double t[3];
};

__device__ inline void load_xform(Xform &X, int b, const float *centers, const float *quats,
                                  const float *translations)
{
    // the ten floats of the pose are requested together (absent arrays read a dummy that is
    // there, then take their default): one trip to memory instead of up to ten
    const float *any = quats ? quats : (centers ? centers : translations);
    const float *q4 = quats ? quats + 4 * b : any;
    const float *c3 = centers ? centers + 3 * b : any;
    const float *t3 = translations ? translations + 3 * b : any;
    float qv[4] = {1.0f, 0.0f, 0.0f, 0.0f}, cv[3] = {0.0f, 0.0f, 0.0f}, tv[3] = {0.0f, 0.0f, 0.0f};
    if (any) {
        for (int m = 0; m < 4; ++m) qv[m] = q4[quats ? m : 0];
        for (int m = 0; m < 3; ++m) cv[m] = c3[centers ? m : 0];
        for (int m = 0; m < 3; ++m) tv[m] = t3[translations ? m : 0];
        asm volatile("" ::"s"(qv[0]), "s"(qv[1]), "s"(qv[2]), "s"(qv[3]), "s"(cv[0]), "s"(cv[1]),
                     "s"(cv[2]), "s"(tv[0]), "s"(tv[1]), "s"(tv[2]));
    }
    const double w = quats ? (double)qv[0] : 1.0, x = quats ? (double)qv[1] : 0.0,
                 y = quats ? (double)qv[2] : 0.0, z = quats ? (double)qv[3] : 0.0;
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
        X.c[m] = centers ? (double)cv[m] : 0.0;
        X.t[m] = translations ? (double)tv[m] : 0.0;
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

// the inverse map, same precision and rounding:  x = R^T ((x' - t) - c) + c
__device__ inline void apply_xform_inverse(const Xform &X, const float *p, float *o)
{
    const double u0 = ((double)p[0] - X.t[0]) - X.c[0];
    const double u1 = ((double)p[1] - X.t[1]) - X.c[1];
    const double u2 = ((double)p[2] - X.t[2]) - X.c[2];
    o[0] = (float)(((X.R[0] * u0 + X.R[3] * u1) + X.R[6] * u2) + X.c[0]);
    o[1] = (float)(((X.R[1] * u0 + X.R[4] * u1) + X.R[7] * u2) + X.c[1]);
    o[2] = (float)(((X.R[2] * u0 + X.R[5] * u1) + X.R[8] * u2) + X.c[2]);
}

}  // namespace mg
