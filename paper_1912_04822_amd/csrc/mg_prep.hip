// Steps 1 and 2 of the path: per-example coordinate transform, radius lookup,
// bounding-box culling, channel binning and x-plane binning.
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
//
// Usual sizes: one workgroup per example (512 threads up to 2048 atoms of index
// types, 1024 otherwise) does a counting sort of the example's atoms by (type, x-plane bin) in LDS:
//   1. every atom: transform, cull, key = type * bins + bin (bins 0 and D+1 are
//      the atoms left / right of the grid, bin D+2 the culled ones), count;
//   2. exclusive scan of the counts = where each (type, bin) starts;
//   3. atoms are placed, each bin is put in atom order (so the order in which
//      the forward kernel sums is fixed), records are written bin by bin;
//   4. for every type and x-plane, the span of records that can reach it.
// N > 8192 or very many (type, bin) pairs take the slower kernel below it: one
// wavefront per group (example b, type t; vector types: example b) that scans
// the example's types for its own atoms.
#include "mg_common.h"
#include "mg_wave.h"
#include "mg_xform.h"

namespace mg {

namespace {

constexpr int kPrepThreads = 64;
constexpr int kMaxBins = 1028;      // MG_MAX_POINTS + 2, rounded up

template <bool INVERSE>
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
    if (INVERSE)
        apply_xform_inverse(X, coords + k, o);
    else
        apply_xform(X, coords + k, o);
    out[k + 0] = o[0];
    out[k + 1] = o[1];
    out[k + 2] = o[2];
}

// Exclusive prefix sum of `v` over the 64 lanes of the wavefront; *total gets the sum.
// (DPP row shifts and broadcasts: no trips through LDS.)
__device__ inline int wave_exclusive_scan(int v, int *total)
{
    const int incl = wave_inclusive_scan(v);
    *total = __builtin_amdgcn_readlane(incl, 63);
    return incl - v;
}

struct Culler {
    float org[3];       // grid origin (center - half)
    float span;         // (D-1)*res
    float pad;
};

// Centre of the grid of virtual example b (source example bs); X holds bs's centre (a float
// widened to double, so narrowing it back is exact).
__device__ inline void grid_center(const Subgrids &sub, const Xform &X, int b, int bs, float *gc)
{
    for (int m = 0; m < 3; ++m) gc[m] = (float)X.c[m];
    if (sub.per_side > 1) {
        const int s = b - bs * sub.count;
        const int sxy = s / sub.per_side;
        const int sv[3] = {sxy / sub.per_side, sxy % sub.per_side, s % sub.per_side};
        for (int m = 0; m < 3; ++m) gc[m] = gc[m] + ((float)sv[m] - sub.mid) * sub.step;
    }
}

// Transformed position, radius and liveness of atom a of (source) example b.
template <bool VECTOR>
__device__ inline bool place_atom(const GridSpec &gs, const Batch &bt, const Xform &X,
                                  const Culler &cu, int b, int t, int a, float vec_reach,
                                  float *p, float *r_out)
{
    apply_xform(X, bt.coords + ((size_t)b * bt.N + a) * 3, p);
    float r, reach;
    if (VECTOR) {
        r = 1.0f;
        reach = vec_reach;
    } else {
        const float rad = gs.radius_type_indexed ? bt.radii[t] : bt.radii[(size_t)b * bt.N + a];
        r = gs.radius_scale * rad;
        reach = gs.binary ? r : r * gs.c;
    }
    bool live = (r > 0.0f) && (reach < 1.0e30f);
    for (int k = 0; k < 3; ++k)     // also false for NaN / infinite coordinates
        live = live && (p[k] >= cu.org[k] - reach - cu.pad) &&
               (p[k] <= cu.org[k] + cu.span + reach + cu.pad);
    *r_out = r;
    return live;
}


// Vector types: the channels of (virtual) example b in order of radius, for the kernels that
// take several channels of an atom together (thread `tid` of `nthreads`).  NaN and negative
// radii rank as 0, so the result is a permutation whatever the table holds.
__device__ inline void rank_channels(const Batch &bt, const Workspace &ws, int b, int tid, int nthreads)
{
    const int T = bt.T;
    for (int k = tid; k < T; k += nthreads) {
        int rank = k;
        if (T <= kRankCap) {
            float mine = bt.radii[k];
            mine = mine > 0.0f ? mine : 0.0f;
            rank = 0;
            for (int j = 0; j < T; ++j) {
                float other = bt.radii[j];
                other = other > 0.0f ? other : 0.0f;
                rank += (other < mine || (other == mine && j < k)) ? 1 : 0;
            }
        }
        ws.chan_order[(size_t)b * T + rank] = k;
    }
}

// ---------------------------------------------------------------------------
// One workgroup per example: counting sort by (type, x-bin) in LDS.
// ---------------------------------------------------------------------------
constexpr int kExThreads = 1024;            // the larger of the two block sizes
constexpr int kExMaxAtoms = 8192;           // 8 atoms per thread (4 in the kernel for N <= 4096)
constexpr int kExMaxKeys = 12288;

struct ExLayout {       // LDS, in ints
    int K, Tg, N;
    __host__ __device__ int cnt() const { return 0; }
    __host__ __device__ int pos() const { return K; }
    __host__ __device__ int rmax() const { return 2 * K; }
    __host__ __device__ int rad() const { return 2 * K + Tg; }                  // float[Tg]
    __host__ __device__ int part() const { return 2 * K + 2 * Tg; }
    __host__ __device__ int order() const { return 2 * K + 2 * Tg + 32; }       // ushort[N]
    __host__ __device__ int ints() const { return order() + (N + 1) / 2; }
};

template <bool VECTOR, int kPer, int NT>
__global__ __launch_bounds__(NT) void prep_example_kernel(GridSpec gs, Batch bt,
                                                                  Workspace ws, unsigned tag,
                                                                  int stop)
{
    extern __shared__ int s_mem[];
    const int b = blockIdx.x, tid = threadIdx.x;
    const int bs = source_example(bt.sub.count, b);       // whose atoms and pose this (virtual) example reads
    const int N = bt.N, T = bt.T, D = gs.D;
    if (MG_STOP_IS(stop, 1)) return;
    const int Tg = VECTOR ? 1 : T;      // groups per example
    const int nb = D + 3;               // bins per group; bin D+2 holds the culled atoms
    ExLayout L;
    L.K = Tg * nb; L.Tg = Tg; L.N = N;
    const int K = L.K;
    int *s_cnt = s_mem + L.cnt();
    int *s_pos = s_mem + L.pos();
    int *s_rmax = s_mem + L.rmax();
    float *s_rad = reinterpret_cast<float *>(s_mem + L.rad());
    int *s_part = s_mem + L.part();
    unsigned short *s_order = reinterpret_cast<unsigned short *>(s_mem + L.order());

    // Everything this thread needs from HBM is requested before anything is waited for:
    // its atoms (thread tid owns atoms tid, tid + 1024, ...), the radii table, the pose.
    const int32_t *ty = VECTOR ? nullptr : bt.types + (size_t)bs * N;
    const float *crd = bt.coords + (size_t)bs * N * 3;          // 32-bit offsets from here on
    const float *rad_b = bt.radii + ((!VECTOR && !gs.radius_type_indexed) ? (size_t)bs * N : 0);
    int my_t[kPer];
    float my_c[kPer][3], my_r[kPer];
#pragma unroll
    for (int u = 0; u < kPer; ++u) {
        const int a = tid + u * NT;
        my_t[u] = -1;
        my_c[u][0] = 0.0f; my_c[u][1] = 0.0f; my_c[u][2] = 0.0f;
        my_r[u] = 0.0f;
        if (a < N) {
            my_t[u] = VECTOR ? 0 : ty[a];
            my_c[u][0] = crd[a * 3];
            my_c[u][1] = crd[a * 3 + 1];
            my_c[u][2] = crd[a * 3 + 2];
            if (!VECTOR && !gs.radius_type_indexed) my_r[u] = rad_b[a];
        }
    }
    // (the radius table too: this thread's entry now, into LDS once the loads have landed)
    const bool rad_table = !VECTOR && gs.radius_type_indexed;
    float my_rad = 0.0f;
    if (rad_table && tid < Tg) my_rad = bt.radii[tid];
    int n = N;
    if (bt.natoms) {
        n = bt.natoms[bs];
        n = n < 0 ? 0 : (n > N ? N : n);
    }
    Xform X;
    load_xform(X, bs, bt.centers, bt.quats, bt.translations);
    if (tid < 9) ws.rot[b * 12 + tid] = (float)X.R[tid];
    if (b == 0 && tid == 0) *ws.tag = tag;
    float vec_reach = 0.0f;         // reach of the widest channel, for vector types
    if (VECTOR) {
        rank_channels(bt, ws, b, tid, NT);
        for (int k = 0; k < T; ++k) {
            const float r = gs.radius_scale * bt.radii[k];
            if (r > vec_reach) vec_reach = r;
        }
        if (!gs.binary) vec_reach *= gs.c;
    }
    Culler cu;
    cu.pad = 1.0e-3f * gs.res;
    cu.span = (float)(D - 1) * gs.res;
    float gc[3];
    grid_center(bt.sub, X, b, bs, gc);
    if (tid < 3) ws.gcen[b * 4 + tid] = gc[tid];
    for (int m = 0; m < 3; ++m) cu.org[m] = gc[m] - gs.half;

    if (rad_table) {
        if (tid < Tg) s_rad[tid] = my_rad;
        for (int k = tid + NT; k < Tg; k += NT) s_rad[k] = bt.radii[k];
    }
    if (MG_STOP_IS(stop, 2)) return;
    for (int k = tid; k < K; k += NT) s_cnt[k] = 0;
    for (int k = tid; k < Tg; k += NT) s_rmax[k] = 0;
    __syncthreads();

    // ---- 1. key and a slot inside its bin for every atom ----
    int my_key[kPer], my_slot[kPer];
    float my_p[kPer][3], my_w[kPer];        // transformed position, radius (0: culled)
#pragma unroll
    for (int u = 0; u < kPer; ++u) {
        const int a = tid + u * NT;
        my_key[u] = 0xFFFF;
        my_slot[u] = 0;
        my_w[u] = 0.0f;
        my_p[u][0] = 0.0f; my_p[u][1] = 0.0f; my_p[u][2] = 0.0f;
        if (a >= N) continue;
        const int tg = my_t[u];
        const bool member = a < n && tg >= 0 && tg < Tg;
        if (member) {
            apply_xform(X, my_c[u], my_p[u]);
            float r, reach;
            if (VECTOR) {
                r = 1.0f;
                reach = vec_reach;
            } else {
                r = gs.radius_scale * (gs.radius_type_indexed ? s_rad[tg] : my_r[u]);
                reach = gs.binary ? r : r * gs.c;
            }
            bool live = (r > 0.0f) && (reach < 1.0e30f);
            for (int k = 0; k < 3; ++k)     // also false for NaN / infinite coordinates
                live = live && (my_p[u][k] >= cu.org[k] - reach - cu.pad) &&
                       (my_p[u][k] <= cu.org[k] + cu.span + reach + cu.pad);
            int bin = D + 2;
            if (live) {
                const float f = floorf((my_p[u][0] - cu.org[0]) * gs.inv_res);
                bin = f < 0.0f ? 0 : (f >= (float)D ? D + 1 : (int)f + 1);
                atomicMax(&s_rmax[tg], __float_as_int(r));      // r > 0: ordered like ints
                my_w[u] = r;
            }
            my_key[u] = tg * nb + bin;
            my_slot[u] = atomicAdd(&s_cnt[my_key[u]], 1);
            ws.alive[(size_t)b * N + a] = live ? 1 : 0;
        } else {
            ws.alive[(size_t)b * N + a] = 0;        // no group owns this atom
        }
    }
    __syncthreads();
    if (MG_STOP_IS(stop, 3)) return;

    // ---- 2. exclusive scan of the counts ----
    const int chunk = (K + NT - 1) / NT;
    const int k0 = min(K, tid * chunk), k1 = min(K, k0 + chunk);
    int mine = 0;
    for (int k = k0; k < k1; ++k) mine += s_cnt[k];
    int wtotal;
    int run = wave_exclusive_scan(mine, &wtotal);
    if ((tid & 63) == 0) s_part[tid >> 6] = wtotal;
    __syncthreads();
    if (tid < 64) {
        int t16;
        const int v = tid < NT / 64 ? s_part[tid] : 0;
        const int ex = wave_exclusive_scan(v, &t16);
        if (tid < NT / 64) s_part[tid] = ex;
        if (tid == 0) s_part[NT / 64] = t16;
    }
    __syncthreads();
    run += s_part[tid >> 6];
    const int total = s_part[NT / 64];      // atoms that belong to a group
    for (int k = k0; k < k1; ++k) {
        s_pos[k] = run;
        run += s_cnt[k];
    }
    __syncthreads();
    if (MG_STOP_IS(stop, 4)) return;

    // ---- 3. atoms into their bins in any order; group descriptors and spans meanwhile ----
#pragma unroll
    for (int u = 0; u < kPer; ++u)
        if (my_key[u] != 0xFFFF) s_order[s_pos[my_key[u]] + my_slot[u]] = (unsigned short)(tid + u * NT);
    for (int tg = tid; tg < Tg; tg += NT) {
        const int first = s_pos[tg * nb];
        const int dead = s_pos[tg * nb + D + 2];
        const int end = tg + 1 < Tg ? s_pos[(tg + 1) * nb] : total;
        ws.meta[(size_t)b * T + tg] = make_int4(first, dead - first, end - first, 1);
    }
    for (int e = tid; e < Tg * D; e += NT) {
        const int tg = e / D, i = e - tg * D;
        // plane i is reached from bins [i - Rv, i + Rv + 1]
        const float rmax = VECTOR ? vec_reach
                                  : __int_as_float(s_rmax[tg]) * (gs.binary ? 1.0f : gs.c);
        const int Rv = (int)ceilf(rmax * gs.inv_res + cu.pad) + 1;
        const int lo = max(0, i - Rv), hi = min(D + 1, i + Rv + 1);
        ws.range[((size_t)b * T + tg) * D + i] = make_int2(s_pos[tg * nb + lo], s_pos[tg * nb + hi + 1]);
    }
    __syncthreads();
    if (MG_STOP_IS(stop, 5)) return;

    // ---- 4. every atom writes its record where its rank inside the bin puts it ----
    // (rank = how many atoms of the bin have a smaller index: the order in which the
    // forward kernel sums is fixed; the order of culled atoms does not matter)
#pragma unroll
    for (int u = 0; u < kPer; ++u) {
        const int key = my_key[u];
        if (key == 0xFFFF) continue;
        const int a = tid + u * NT;
        const int lo = s_pos[key];
        int rank = my_slot[u];
        if (key - (key / nb) * nb != D + 2) {
            const int cnt = s_cnt[key];
            rank = 0;
            for (int i = 0; i < cnt; ++i) rank += s_order[lo + i] < a ? 1 : 0;
        }
        ws.rec[(size_t)b * N + lo + rank] = make_float4(my_p[u][0], my_p[u][1], my_p[u][2], my_w[u]);
        ws.idx[(size_t)b * N + lo + rank] = a;
        if (!VECTOR) ws.rchan[(size_t)b * N + lo + rank] = key / nb;
    }
}

// One wavefront per group: no barriers, the scans are wavefront shuffles.
template <bool VECTOR>
__global__ __launch_bounds__(64) void prep_kernel(GridSpec gs, Batch bt, Workspace ws,
                                                  unsigned tag, int stop)
{
    __shared__ int s_list[kSortCap];                // atom index of match m
    __shared__ unsigned short s_bin[kSortCap];      // x-bin of match m, 0xFFFF = culled
    __shared__ unsigned short s_order[kSortCap];    // match id at sorted position
    __shared__ int s_cnt[kMaxBins];                 // records per bin
    __shared__ int s_pos[kMaxBins];                 // start of bin, then fill cursor
    __shared__ int s_rmax;

    const int b = blockIdx.y, t = blockIdx.x, lane = threadIdx.x;
    const int bs = source_example(bt.sub.count, b);       // whose atoms and pose this (virtual) example reads
    const int N = bt.N, T = bt.T, D = gs.D;
    if (MG_STOP_IS(stop, 1)) return;
    int n = N;
    if (bt.natoms) {
        n = bt.natoms[bs];
        n = n < 0 ? 0 : (n > N ? N : n);
    }
    const int32_t *ty = VECTOR ? nullptr : bt.types + (size_t)bs * N;

    Xform X;
    load_xform(X, bs, bt.centers, bt.quats, bt.translations);

    // ---- 1. stable compaction: lane owns atoms [a0, a1) ----
    const int per = (n + 63) / 64;
    const int a0 = min(n, lane * per), a1 = min(n, a0 + per);
    int less = 0, eq = 0;
    unsigned long long eqmask = 0ull;       // matches among the first 64 atoms of the run
    if (VECTOR) {
        eq = a1 - a0;
    } else {
        for (int c0 = a0; c0 < a1; c0 += 16) {
            int v[16];
#pragma unroll
            for (int u = 0; u < 16; ++u) v[u] = (c0 + u < a1) ? ty[c0 + u] : -1;
#pragma unroll
            for (int u = 0; u < 16; ++u) {
                less += (v[u] >= 0 && v[u] < t) ? 1 : 0;
                if (v[u] == t) {
                    ++eq;
                    if (c0 - a0 + u < 64) eqmask |= 1ull << (c0 - a0 + u);
                }
            }
        }
    }
    if (MG_STOP_IS(stop, 2)) { if (less + eq == 12345) ws.rot[0] = 1.0f; return; }
    int M, first;
    const int my_first = wave_exclusive_scan(eq, &M);
    (void)wave_exclusive_scan(less, &first);
    if (VECTOR) first = 0;
    if (t == 0 && lane < 9) ws.rot[b * 12 + lane] = (float)X.R[lane];
    if (VECTOR) rank_channels(bt, ws, b, lane, kPrepThreads);      // (one wavefront per example)
    if (MG_STOP_IS(stop, 3)) { if (M + first == 12345) ws.rot[0] = 1.0f; return; }

    float vec_reach = 0.0f;         // reach of the widest channel, for vector types
    if (VECTOR) {
        for (int k = 0; k < T; ++k) {
            const float r = gs.radius_scale * bt.radii[k];
            if (r > vec_reach) vec_reach = r;
        }
        if (!gs.binary) vec_reach *= gs.c;
    }
    Culler cu;
    cu.pad = 1.0e-3f * gs.res;
    cu.span = (float)(D - 1) * gs.res;
    float gc[3];
    grid_center(bt.sub, X, b, bs, gc);
    if (t == 0 && lane < 3) ws.gcen[b * 4 + lane] = gc[lane];
    for (int m = 0; m < 3; ++m) cu.org[m] = gc[m] - gs.half;

    float4 *rec = ws.rec + (size_t)b * N + first;
    int *idx = ws.idx + (size_t)b * N + first;
    int *rchan = ws.rchan + (size_t)b * N + first;
    const size_t group = (size_t)b * T + t;
    const int nbins = D + 2;

    if (M <= kSortCap) {
        // ---- 2. match list, transform, cull, count per x-bin ----
        for (int k = lane; k < nbins; k += 64) s_cnt[k] = 0;
        if (lane == 0) s_rmax = 0;
        int rank = my_first;
        if (VECTOR) {
            for (int a = a0; a < a1; ++a) s_list[rank++] = a;
        } else {
            unsigned long long mk = eqmask;
            while (mk != 0ull) {
                s_list[rank++] = a0 + (int)__builtin_ctzll(mk);
                mk &= mk - 1ull;
            }
            for (int a = a0 + 64; a < a1; ++a)
                if (ty[a] == t) s_list[rank++] = a;
        }
        lds_sync();
        for (int m = lane; m < M; m += 64) {
            const int a = s_list[m];
            float p[3], r;
            const bool live = place_atom<VECTOR>(gs, bt, X, cu, bs, t, a, vec_reach, p, &r);
            int bin = 0xFFFF;
            if (live) {
                const float f = floorf((p[0] - cu.org[0]) * gs.inv_res);
                bin = f < 0.0f ? 0 : (f >= (float)D ? D + 1 : (int)f + 1);
                atomicAdd(&s_cnt[bin], 1);
                atomicMax(&s_rmax, __float_as_int(r));      // r > 0: ordered like ints
            }
            ws.alive[(size_t)b * N + a] = live ? 1 : 0;
            s_bin[m] = (unsigned short)bin;
        }
        lds_sync();
        if (MG_STOP_IS(stop, 4)) return;
        // ---- 3. bin starts (exclusive scan over the bins) ----
        const int bper = (nbins + 63) / 64;
        const int k0 = min(nbins, lane * bper), k1 = min(nbins, k0 + bper);
        int mine = 0;
        for (int k = k0; k < k1; ++k) mine += s_cnt[k];
        int L;
        int run = wave_exclusive_scan(mine, &L);
        for (int k = k0; k < k1; ++k) {
            s_pos[k] = run;
            run += s_cnt[k];
        }
        lds_sync();
        // ---- 4. span of records that can reach each plane ----
        // plane i is reached from bins [i - Rv, i + Rv + 1]
        const float rmax = VECTOR ? vec_reach : __int_as_float(s_rmax) * (gs.binary ? 1.0f : gs.c);
        const int Rv = (int)ceilf(rmax * gs.inv_res + cu.pad) + 1;
        for (int i = lane; i < D; i += 64) {
            const int lo = max(0, i - Rv), hi = min(D + 1, i + Rv + 1);
            ws.range[group * D + i] = make_int2(first + s_pos[lo], first + (hi + 1 < nbins ? s_pos[hi + 1] : L));
        }
        lds_sync();
        if (MG_STOP_IS(stop, 5)) return;
        // ---- 5. placement: any order inside a bin, then sort each bin by atom order ----
        for (int m = lane; m < M; m += 64) {
            const int bin = s_bin[m];
            if (bin != 0xFFFF) s_order[atomicAdd(&s_pos[bin], 1)] = (unsigned short)m;
        }
        lds_sync();
        for (int k = lane; k < nbins; k += 64) {
            const int hi = s_pos[k], lo = hi - s_cnt[k];
            for (int i = lo + 1; i < hi; ++i) {
                const unsigned short v = s_order[i];
                int j = i - 1;
                while (j >= lo && s_order[j] > v) {
                    s_order[j + 1] = s_order[j];
                    --j;
                }
                s_order[j + 1] = v;
            }
        }
        lds_sync();
        if (MG_STOP_IS(stop, 6)) return;
        // ---- 6. records in sorted order (the transform is cheap: done again) ----
        for (int pos = lane; pos < M; pos += 64) {
            if (pos < L) {
                const int a = s_list[s_order[pos]];
                float p[3], r;
                (void)place_atom<VECTOR>(gs, bt, X, cu, bs, t, a, vec_reach, p, &r);
                rec[pos] = make_float4(p[0], p[1], p[2], r);
                idx[pos] = a;
                rchan[pos] = t;
            } else {
                rec[pos] = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
                idx[pos] = -1;
                rchan[pos] = t;
            }
        }
        if (lane == 0) ws.meta[group] = make_int4(first, L, M, 1);
    } else {
        // ---- group too long to bin: records in atom order, culled ones flagged r = 0 ----
        for (int r0 = 0; r0 < M; r0 += kSortCap) {
            int rank = my_first;
            for (int a = a0; a < a1; ++a) {
                if (VECTOR || ty[a] == t) {
                    if (rank >= r0 && rank < r0 + kSortCap) s_list[rank - r0] = a;
                    ++rank;
                }
            }
            lds_sync();
            const int cnt = min(kSortCap, M - r0);
            for (int m = lane; m < cnt; m += 64) {
                const int a = s_list[m];
                float p[3], r;
                const bool live = place_atom<VECTOR>(gs, bt, X, cu, bs, t, a, vec_reach, p, &r);
                rec[r0 + m] = make_float4(p[0], p[1], p[2], live ? r : 0.0f);
                idx[r0 + m] = a;
                rchan[r0 + m] = t;
                ws.alive[(size_t)b * N + a] = live ? 1 : 0;
            }
            lds_sync();
        }
        for (int i = lane; i < D; i += 64) ws.range[group * D + i] = make_int2(first, first + M);
        if (lane == 0) ws.meta[group] = make_int4(first, M, M, 0);
    }

    // atoms no group owns (past natoms, type outside [0,T)) are not alive
    if (t == 0) {
        for (int a = lane; a < N; a += 64) {
            bool orphan = a >= n;
            if (!VECTOR && !orphan) {
                const int v = ty[a];
                orphan = v < 0 || v >= T;
            }
            if (orphan) ws.alive[(size_t)b * N + a] = 0;
        }
        if (b == 0 && lane == 0) *ws.tag = tag;
    }
}

size_t align16(size_t v) { return (v + 15) / 16 * 16; }

}  // namespace

size_t workspace_bytes(const GridSpec &gs, int subgrid_count, int B, int N, int T)
{
    const size_t bn = (size_t)B * (size_t)N, bt = (size_t)B * (size_t)T;
    size_t bytes = bn * sizeof(float4);                     // rec
    bytes += align16(bn * sizeof(int));                     // idx
    bytes += bt * sizeof(int4);                             // meta
    bytes += align16(bt * (size_t)gs.D * sizeof(int2));     // range
    bytes += (size_t)B * 12 * sizeof(float);                // rot
    bytes += (size_t)B * 4 * sizeof(float);                 // gcen
    bytes += align16(bt * sizeof(int));                     // chan_order
    bytes += align16(bn);                                   // alive
    bytes += align16(bn * sizeof(int));                     // rchan
    bytes += 16;                                            // tag
    if (subgrid_count > 1) {
        bytes += align16(bn * 3 * sizeof(float));           // gtmp
        if (gs.radius_type_indexed) bytes += align16(bn * (size_t)T * sizeof(float));   // wtmp
    }
    return bytes;
}

Workspace carve_workspace(const GridSpec &gs, int subgrid_count, void *base, int B, int N, int T)
{
    const size_t bn = (size_t)B * (size_t)N, bt = (size_t)B * (size_t)T;
    char *p = (char *)base;
    Workspace ws;
    ws.rec = (float4 *)p;
    p += bn * sizeof(float4);
    ws.idx = (int *)p;
    p += align16(bn * sizeof(int));
    ws.meta = (int4 *)p;
    p += bt * sizeof(int4);
    ws.range = (int2 *)p;
    p += align16(bt * (size_t)gs.D * sizeof(int2));
    ws.rot = (float *)p;
    p += (size_t)B * 12 * sizeof(float);
    ws.gcen = (float *)p;
    p += (size_t)B * 4 * sizeof(float);
    ws.chan_order = (int *)p;
    p += align16(bt * sizeof(int));
    ws.alive = (unsigned char *)p;
    p += align16(bn);
    ws.rchan = (int *)p;
    p += align16(bn * sizeof(int));
    ws.tag = (unsigned *)p;
    p += 16;
    ws.gtmp = nullptr;
    ws.wtmp = nullptr;
    if (subgrid_count > 1) {
        ws.gtmp = (float *)p;
        p += align16(bn * 3 * sizeof(float));
        if (gs.radius_type_indexed) ws.wtmp = (float *)p;
    }
    return ws;
}

hipError_t launch_transform(int B, int N, const float *coords, const float *centers,
                            const float *quats, const float *translations, float *out,
                            bool inverse, hipStream_t stream)
{
    dim3 grid((N + 255) / 256, B);
    if (inverse)
        hipLaunchKernelGGL(transform_kernel<true>, grid, dim3(256), 0, stream, B, N, coords,
                           centers, quats, translations, out);
    else
        hipLaunchKernelGGL(transform_kernel<false>, grid, dim3(256), 0, stream, B, N, coords,
                           centers, quats, translations, out);
    return hipGetLastError();
}

// What the tables were made for, folded into one word (never 0): the kernels of a *_prepared
// call compare it with their own arguments and do nothing if the workspace holds something else.
unsigned workspace_tag(const GridSpec &gs, const Batch &bt)
{
    unsigned long long h = 0x9E3779B97F4A7C15ull;
    const unsigned words[] = {(unsigned)bt.B, (unsigned)bt.N, (unsigned)bt.T, (unsigned)gs.D,
                              (unsigned)bt.sub.per_side, bt.vec ? 1u : 0u, (unsigned)gs.binary,
                              (unsigned)gs.radius_type_indexed};
    for (unsigned w : words) {
        h ^= w;
        h *= 0x100000001B3ull;
        h ^= h >> 29;
    }
    const unsigned t = (unsigned)(h ^ (h >> 32));
    return t ? t : 1u;
}

hipError_t launch_prep(const GridSpec &gs, const Batch &bt, const Workspace &ws, int stop,
                       hipStream_t stream)
{
    const unsigned tag = workspace_tag(gs, bt);
    const bool vec = bt.vec;
    ExLayout L;
    L.Tg = vec ? 1 : bt.T;
    L.N = bt.N;
    const long long K = (long long)L.Tg * (gs.D + 3);
    L.K = (int)(K <= kExMaxKeys ? K : 0);
    const size_t lds_bytes = (size_t)L.ints() * sizeof(int);
    if (K <= kExMaxKeys && bt.N <= kExMaxAtoms && lds_bytes <= 64 * 1024) {
        const dim3 grd(bt.B);
        // 512 threads while they still hold all the atoms four apiece: half as many wavefronts
        // behind every barrier (1 us less per call at 2040 atoms; 256 threads with eight atoms
        // apiece measured 4 us more)
        if (bt.N <= 4 * 512 && !vec) {      // (vector types, which also rank the channels: 1024 is 1.5 us quicker)
            hipLaunchKernelGGL((prep_example_kernel<false, 4, 512>), grd, dim3(512), lds_bytes, stream, gs,
                               bt, ws, tag, stop);
            return hipGetLastError();
        }
        const dim3 blk(kExThreads);
        if (bt.N <= 4 * kExThreads) {
            if (vec)
                hipLaunchKernelGGL((prep_example_kernel<true, 4, kExThreads>), grd, blk, lds_bytes, stream, gs, bt,
                                   ws, tag, stop);
            else
                hipLaunchKernelGGL((prep_example_kernel<false, 4, kExThreads>), grd, blk, lds_bytes, stream, gs,
                                   bt, ws, tag, stop);
        } else {
            if (vec)
                hipLaunchKernelGGL((prep_example_kernel<true, 8, kExThreads>), grd, blk, lds_bytes, stream, gs, bt,
                                   ws, tag, stop);
            else
                hipLaunchKernelGGL((prep_example_kernel<false, 8, kExThreads>), grd, blk, lds_bytes, stream, gs,
                                   bt, ws, tag, stop);
        }
        return hipGetLastError();
    }
    if (vec) {
        hipLaunchKernelGGL(prep_kernel<true>, dim3(1, bt.B), dim3(kPrepThreads), 0, stream, gs, bt,
                           ws, tag, stop);
    } else {
        hipLaunchKernelGGL(prep_kernel<false>, dim3(bt.T, bt.B), dim3(kPrepThreads), 0, stream, gs,
                           bt, ws, tag, stop);
    }
    return hipGetLastError();
}

}  // namespace mg
