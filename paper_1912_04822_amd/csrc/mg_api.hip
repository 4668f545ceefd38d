// The C ABI (include/molgrid_hip.h): argument validation on the host, then the
// launches.  No allocation, no synchronisation, no host<->device copies.
#include "../../include/molgrid_hip.h"

#include <atomic>
#include <cmath>
#include <cstring>
#include <new>

#include "mg_common.h"

struct mg_gridmaker {
    mg::GridSpec gs;
    mg::Subgrids sub;
    float dimension;
    float grm;
};

// The workspace of mg_forward_index_static: one array per GPU, held until the process ends.
// The name is a host-side stand-in, not a device address: host code only ever uses the
// per-device address hipGetSymbolAddress returned (static_scratch below).
static __device__ __align__(256) unsigned char scratch[MG_STATIC_WORKSPACE_BYTES];

namespace {

thread_local int g_last_hip_error = 0;
thread_local hipEvent_t g_ev_start = nullptr, g_ev_stop = nullptr;
// Launch knobs (mg_set_option): process-wide, read once per call.  Atomic so that a thread
// that sets one while another thread makes a call is a defined (if unordered) program.
std::atomic<int> g_tile_floats{0};       // 0: chosen by the launcher
std::atomic<int> g_waves_per_tile{0};    // 0: chosen by the launcher
std::atomic<int> g_xcd_run{0};
std::atomic<int> g_lds_floor{-1};        // < 0: chosen by the launcher
std::atomic<int> g_tile_order{0};
std::atomic<int> g_keep_alive{1};
std::atomic<int> g_keep_alive_stride{1};
std::atomic<int> g_single_launch{1};     // small problems: the forward kernel alone, no prep kernel
#ifdef MG_TIMING_AIDS
std::atomic<int> g_debug{0};             // measurement build only: kernel phases switched off
std::atomic<int> g_prep_stop{0};         // measurement build only: prep kernel ended after a stage
#endif

int timing_debug()
{
#ifdef MG_TIMING_AIDS
    return g_debug.load(std::memory_order_relaxed);
#else
    return 0;
#endif
}

int timing_prep_stop()
{
#ifdef MG_TIMING_AIDS
    return g_prep_stop.load(std::memory_order_relaxed);
#else
    return 0;
#endif
}

// The caller's timing events for the main kernel of this call, if set (cleared by the call).
mg::KernelEvents take_events()
{
    mg::KernelEvents ev = {g_ev_start, g_ev_stop};
    g_ev_start = nullptr;
    g_ev_stop = nullptr;
    return ev;
}

constexpr int kMaxDevices = 64;
std::atomic<void *> g_scratch_ptr[kMaxDevices];

// Address of `scratch` on the current device, looked up once per device (each GPU holds its
// own copy of the array at its own address).  Two threads racing here store the same value.
int static_scratch(void **ptr, int *hip_error)
{
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess || dev < 0 || dev >= kMaxDevices) {
        *hip_error = (int)(e != hipSuccess ? e : hipErrorInvalidDevice);
        return MG_EHIP;
    }
    void *p = g_scratch_ptr[dev].load(std::memory_order_acquire);
    if (!p) {
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !p) {
            *hip_error = (int)(e != hipSuccess ? e : hipErrorInvalidSymbol);
            return MG_EHIP;
        }
        g_scratch_ptr[dev].store(p, std::memory_order_release);
    }
    *ptr = p;
    return MG_OK;
}

bool finite_pos(float v) { return std::isfinite(v) && v > 0.0f; }

int check_shape(const mg_gridmaker *gm, int B, int N, int T)
{
    if (!gm) return MG_ENULL;
    if (B < 1 || N < 1 || T < 1) return MG_ESHAPE;
    if (B > 65535 / gm->sub.count) return MG_ESHAPE;        // B below counts virtual examples
    B *= gm->sub.count;
    if (B > 65535 || T > 65535) return MG_ESHAPE;         // grid.y, grid.z of the launches
    const long long D = gm->gs.D;
    const long long tiles = (long long)B * T * ((D * D * D + 511) / 512);   // forward workgroups
    if (tiles > 0x7fffffffLL) return MG_ESHAPE;
    if ((long long)B * T * D * D > 0x7fffffffLL) return MG_ESHAPE;
    if ((long long)B * N > 0x7fffffffLL / 32) return MG_ESHAPE;
    return MG_OK;
}

int check_workspace(const mg_gridmaker *gm, int B, int N, int T, void *ws, size_t ws_bytes)
{
    if (!ws) return MG_EWORKSPACE;
    if (((uintptr_t)ws & 31u) != 0) return MG_EWORKSPACE;
    if (ws_bytes < mg::workspace_bytes(gm->gs, gm->sub.count, B * gm->sub.count, N, T)) return MG_EWORKSPACE;
    return MG_OK;
}

bool misaligned4(const void *p) { return p && (((uintptr_t)p & 3u) != 0); }

int hip_status(hipError_t e)
{
    if (e == hipSuccess) return MG_OK;
    g_last_hip_error = (int)e;
    return MG_EHIP;
}

// B: the caller's examples; the batch counts virtual examples (subgrids).
mg::Batch make_batch(const mg_gridmaker *gm, int B, int N, int T, const float *coords, const int32_t *types,
                     const float *weights, const float *radii, const int32_t *natoms,
                     const float *centers, const float *quats, const float *translations)
{
    mg::Batch bt;
    bt.B = B * gm->sub.count; bt.N = N; bt.T = T;
    bt.sub = gm->sub;
    bt.vec = types == nullptr;      // index types have their type array; everything else is vector types
    bt.coords = coords; bt.types = types; bt.weights = weights; bt.radii = radii;
    bt.natoms = natoms; bt.centers = centers; bt.quats = quats; bt.translations = translations;
    return bt;
}

}  // namespace

extern "C" {

int mg_gridmaker_create(mg_gridmaker **out, float resolution, float dimension, int binary,
                        int radius_type_indexed, float radius_scale, float gaussian_radius_multiple)
{
    return mg_gridmaker_create_subgrids(out, resolution, dimension, 1, binary, radius_type_indexed,
                                        radius_scale, gaussian_radius_multiple);
}

int mg_gridmaker_create_subgrids(mg_gridmaker **out, float resolution, float dimension,
                                 int subgrids_per_side, int binary, int radius_type_indexed,
                                 float radius_scale, float gaussian_radius_multiple)
{
    if (!out) return MG_ENULL;
    if (subgrids_per_side < 1 || subgrids_per_side > MG_MAX_SUBGRIDS) return MG_ESHAPE;
    if (!finite_pos(resolution) || !std::isfinite(dimension) || dimension < 0.0f ||
        !finite_pos(radius_scale) || !finite_pos(gaussian_radius_multiple))
        return MG_EPARAM;
    const double dd = std::floor((double)dimension / (double)resolution + 0.5) + 1.0;
    if (!(dd >= 1.0) || dd > (double)MG_MAX_POINTS) return MG_ESHAPE;
    mg_gridmaker *gm = new (std::nothrow) mg_gridmaker;
    if (!gm) return MG_ENOMEM;
    const int D = (int)dd;
    const double g = (double)gaussian_radius_multiple;
    const double c = (1.0 + 2.0 * g * g) / (2.0 * g);
    gm->gs.res = resolution;
    gm->gs.half = (float)(0.5 * (D - 1) * (double)resolution);
    gm->gs.inv_res = (float)(1.0 / (double)resolution);
    gm->gs.D = D;
    gm->gs.binary = binary ? 1 : 0;
    gm->gs.radius_type_indexed = radius_type_indexed ? 1 : 0;
    gm->gs.radius_scale = radius_scale;
    gm->gs.g2 = (float)(g * g);
    gm->gs.c = (float)c;
    gm->gs.c2 = (float)(c * c);
    gm->gs.A = (float)(4.0 * g * g * std::exp(-2.0 * g * g));
    gm->sub.per_side = subgrids_per_side;
    gm->sub.count = subgrids_per_side * subgrids_per_side * subgrids_per_side;
    gm->sub.mid = 0.5f * (float)(subgrids_per_side - 1);
    gm->sub.step = (float)D * resolution;
    gm->dimension = dimension;
    gm->grm = gaussian_radius_multiple;
    *out = gm;
    return MG_OK;
}

void mg_gridmaker_destroy(mg_gridmaker *gm) { delete gm; }

int mg_gridmaker_points_per_side(const mg_gridmaker *gm, int *D)
{
    if (!gm || !D) return MG_ENULL;
    *D = gm->gs.D;
    return MG_OK;
}

int mg_gridmaker_subgrids_per_side(const mg_gridmaker *gm, int *S)
{
    if (!gm || !S) return MG_ENULL;
    *S = gm->sub.per_side;
    return MG_OK;
}

int mg_workspace_bytes(const mg_gridmaker *gm, int B, int N, int T, size_t *bytes)
{
    if (!bytes) return MG_ENULL;
    const int rc = check_shape(gm, B, N, T);
    if (rc != MG_OK) return rc;
    *bytes = mg::workspace_bytes(gm->gs, gm->sub.count, B * gm->sub.count, N, T);
    return MG_OK;
}

static int transform_call(int B, int N, const float *coords, const float *centers,
                          const float *quats, const float *translations, float *out,
                          bool inverse, void *stream)
{
    if (!coords || !out) return MG_ENULL;
    if (B < 1 || N < 1 || B > 65535) return MG_ESHAPE;
    if (misaligned4(coords) || misaligned4(out) || misaligned4(centers) || misaligned4(quats) ||
        misaligned4(translations))
        return MG_EALIGN;
    return hip_status(mg::launch_transform(B, N, coords, centers, quats, translations, out,
                                           inverse, (hipStream_t)stream));
}

int mg_transform_forward(int B, int N, const float *coords, const float *centers,
                         const float *quats, const float *translations, float *out, void *stream)
{
    return transform_call(B, N, coords, centers, quats, translations, out, false, stream);
}

int mg_transform_backward(int B, int N, const float *coords, const float *centers,
                          const float *quats, const float *translations, float *out, void *stream)
{
    return transform_call(B, N, coords, centers, quats, translations, out, true, stream);
}

int mg_draw_transforms(uint64_t seed, uint64_t draw, int B, int random_rotation,
                       float max_translation, float *quats, float *translations, void *stream)
{
    if (!quats || !translations) return MG_ENULL;
    if (B < 1 || B > 65535) return MG_ESHAPE;
    if (!(max_translation >= 0.0f) || !std::isfinite(max_translation)) return MG_EPARAM;
    if (misaligned4(quats) || misaligned4(translations)) return MG_EALIGN;
    return hip_status(mg::launch_draw_transforms(seed, draw, B, random_rotation != 0,
                                                 max_translation, quats, translations,
                                                 (hipStream_t)stream));
}

// How a call uses the workspace's tables: builds them and runs (the ordinary calls), builds them
// only (mg_prepare), or runs on tables an earlier call built (the *_prepared calls).
enum class Tables { kBuildAndRun, kBuildOnly, kUseBuilt };

// Forward with either kind of types (types or weights is NULL) into a float or double grid.
// With Tables::kUseBuilt, index types pass `index_types` = true and no arrays but the output
// (the tables hold everything), vector types pass weights and radii.
static int forward_call(const mg_gridmaker *gm, int B, int N, int T, const float *coords,
                        const int32_t *types, const float *weights, const float *radii,
                        const int32_t *natoms, const float *centers, const float *quats,
                        const float *translations, void *out, bool out_is_double, void *workspace,
                        size_t workspace_bytes, void *stream, Tables tables = Tables::kBuildAndRun,
                        bool index_types = false)
{
    if (tables == Tables::kUseBuilt) {
        if (!gm || !out || (!index_types && (!weights || !radii))) return MG_ENULL;
    } else if (tables == Tables::kBuildOnly) {
        if (!gm || !coords || !radii) return MG_ENULL;
    } else {
        if (!gm || !coords || (!types && !weights) || !radii || !out) return MG_ENULL;
    }
    const bool vector_types = tables == Tables::kUseBuilt ? !index_types : types == nullptr;
    if (vector_types && !gm->gs.radius_type_indexed) return MG_EMODE;    // vector types need radii per type
    int rc = check_shape(gm, B, N, T);
    if (rc != MG_OK) return rc;
    if (misaligned4(coords) || misaligned4(types) || misaligned4(weights) || misaligned4(radii) ||
        misaligned4(natoms) || misaligned4(centers) || misaligned4(quats) ||
        misaligned4(translations) || ((uintptr_t)out & (out_is_double ? 7u : 3u)) != 0)
        return MG_EALIGN;
    rc = check_workspace(gm, B, N, T, workspace, workspace_bytes);
    if (rc != MG_OK) return rc;
    mg::Batch bt = make_batch(gm, B, N, T, coords, types, weights, radii, natoms, centers,
                              quats, translations);
    bt.vec = vector_types;
    const mg::Workspace ws = mg::carve_workspace(gm->gs, gm->sub.count, workspace, bt.B, N, T);
    const auto knob = [](const std::atomic<int> &k) { return k.load(std::memory_order_relaxed); };
    const int stop = timing_prep_stop();
    // a few hundred atoms in all: one launch, every tile looks at the atoms itself
    const bool single = tables == Tables::kBuildAndRun && knob(g_single_launch) != 0 && stop == 0 &&
                        timing_debug() == 0 && mg::forward_takes_single_launch(bt, out_is_double);
    if (tables != Tables::kUseBuilt && !single) {
        rc = hip_status(mg::launch_prep(gm->gs, bt, ws, stop, (hipStream_t)stream));
        if (rc != MG_OK || stop != 0) return rc;    // a prep kernel cut short leaves no tables to read
    }
    if (tables == Tables::kBuildOnly) return MG_OK;
    const unsigned expect = tables == Tables::kUseBuilt ? mg::workspace_tag(gm->gs, bt) : 0u;
    return hip_status(mg::launch_forward(gm->gs, bt, ws, out, out_is_double, knob(g_tile_floats),
                                         knob(g_waves_per_tile), knob(g_xcd_run), knob(g_lds_floor),
                                         timing_debug(), knob(g_tile_order), knob(g_keep_alive), single,
                                         expect, take_events(), (hipStream_t)stream,
                                         knob(g_keep_alive_stride)));
}

int mg_prepare(const mg_gridmaker *gm, int B, int N, int T, const float *coords,
               const int32_t *types, const float *radii, const int32_t *natoms,
               const float *centers, const float *quats, const float *translations,
               void *workspace, size_t workspace_bytes, void *stream)
{
    return forward_call(gm, B, N, T, coords, types, nullptr, radii, natoms, centers, quats,
                        translations, nullptr, false, workspace, workspace_bytes, stream,
                        Tables::kBuildOnly);
}

int mg_forward_index_prepared(const mg_gridmaker *gm, int B, int N, int T, float *out,
                              void *workspace, size_t workspace_bytes, void *stream)
{
    return forward_call(gm, B, N, T, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr,
                        nullptr, out, false, workspace, workspace_bytes, stream, Tables::kUseBuilt,
                        true);
}

int mg_forward_vector_prepared(const mg_gridmaker *gm, int B, int N, int T, const float *weights,
                               const float *radii, float *out, void *workspace,
                               size_t workspace_bytes, void *stream)
{
    return forward_call(gm, B, N, T, nullptr, nullptr, weights, radii, nullptr, nullptr, nullptr,
                        nullptr, out, false, workspace, workspace_bytes, stream, Tables::kUseBuilt,
                        false);
}

int mg_forward_index(const mg_gridmaker *gm, int B, int N, int T, const float *coords,
                     const int32_t *types, const float *radii, const int32_t *natoms,
                     const float *centers, const float *quats, const float *translations,
                     float *out, void *workspace, size_t workspace_bytes, void *stream)
{
    if (!types) return MG_ENULL;
    return forward_call(gm, B, N, T, coords, types, nullptr, radii, natoms, centers, quats,
                        translations, out, false, workspace, workspace_bytes, stream);
}

int mg_forward_index_static(const mg_gridmaker *gm, int B, int N, int T, const float *coords,
                            const int32_t *types, const float *radii, const int32_t *natoms,
                            const float *centers, const float *quats, const float *translations,
                            float *out, void *stream)
{
    if (!gm || !types) return MG_ENULL;
    const int rc = check_shape(gm, B, N, T);
    if (rc != MG_OK) return rc;
    if (mg::workspace_bytes(gm->gs, gm->sub.count, B * gm->sub.count, N, T) > (size_t)MG_STATIC_WORKSPACE_BYTES)
        return MG_EWORKSPACE;
    if (!coords || !radii || !out) return MG_ENULL;       // before the device is asked for anything
    void *ws = nullptr;
    int herr = 0;
    if (static_scratch(&ws, &herr) != MG_OK) {
        g_last_hip_error = herr;
        return MG_EHIP;
    }
    return forward_call(gm, B, N, T, coords, types, nullptr, radii, natoms, centers, quats,
                        translations, out, false, ws, (size_t)MG_STATIC_WORKSPACE_BYTES, stream);
}

int mg_forward_index_f64(const mg_gridmaker *gm, int B, int N, int T, const float *coords,
                         const int32_t *types, const float *radii, const int32_t *natoms,
                         const float *centers, const float *quats, const float *translations,
                         double *out, void *workspace, size_t workspace_bytes, void *stream)
{
    if (!types) return MG_ENULL;
    return forward_call(gm, B, N, T, coords, types, nullptr, radii, natoms, centers, quats,
                        translations, out, true, workspace, workspace_bytes, stream);
}

int mg_forward_vector(const mg_gridmaker *gm, int B, int N, int T, const float *coords,
                      const float *weights, const float *radii, const int32_t *natoms,
                      const float *centers, const float *quats, const float *translations,
                      float *out, void *workspace, size_t workspace_bytes, void *stream)
{
    if (!weights) return MG_ENULL;
    return forward_call(gm, B, N, T, coords, nullptr, weights, radii, natoms, centers, quats,
                        translations, out, false, workspace, workspace_bytes, stream);
}

int mg_forward_vector_f64(const mg_gridmaker *gm, int B, int N, int T, const float *coords,
                          const float *weights, const float *radii, const int32_t *natoms,
                          const float *centers, const float *quats, const float *translations,
                          double *out, void *workspace, size_t workspace_bytes, void *stream)
{
    if (!weights) return MG_ENULL;
    return forward_call(gm, B, N, T, coords, nullptr, weights, radii, natoms, centers, quats,
                        translations, out, true, workspace, workspace_bytes, stream);
}

// Backward with either kind of types from a float or double gradient grid.
static int backward_call(const mg_gridmaker *gm, int B, int N, int T, const float *coords,
                         const int32_t *types, const float *weights, const float *radii,
                         const int32_t *natoms, const float *centers, const float *quats,
                         const float *translations, const void *grad_out, bool grad_is_double,
                         float *grad_coords, float *grad_weights, void *workspace,
                         size_t workspace_bytes, void *stream, Tables tables = Tables::kBuildAndRun,
                         bool index_types = false)
{
    if (tables == Tables::kUseBuilt) {      // index types: nothing but the tables; vector types: weights and radii
        if (!gm || (!index_types && (!weights || !radii)) || !grad_out) return MG_ENULL;
    } else {
        if (!gm || !coords || (!types && !weights) || !radii || !grad_out) return MG_ENULL;
        index_types = types != nullptr;
    }
    if (!grad_coords && !grad_weights) return MG_ENULL;
    if (index_types && !grad_coords) return MG_ENULL;
    if (gm->gs.binary || (!index_types && !gm->gs.radius_type_indexed)) return MG_EMODE;
    int rc = check_shape(gm, B, N, T);
    if (rc != MG_OK) return rc;
    if (misaligned4(coords) || misaligned4(types) || misaligned4(weights) || misaligned4(radii) ||
        misaligned4(grad_coords) || misaligned4(grad_weights) || misaligned4(natoms) ||
        misaligned4(centers) || misaligned4(quats) || misaligned4(translations) ||
        ((uintptr_t)grad_out & (grad_is_double ? 7u : 3u)) != 0)
        return MG_EALIGN;
    rc = check_workspace(gm, B, N, T, workspace, workspace_bytes);
    if (rc != MG_OK) return rc;
    mg::Batch bt = make_batch(gm, B, N, T, coords, types, weights, radii, natoms, centers,
                              quats, translations);
    bt.vec = !index_types;
    const mg::Workspace ws = mg::carve_workspace(gm->gs, gm->sub.count, workspace, bt.B, N, T);
    // with subgrids each virtual example's gradient goes to the workspace and they are summed
    const bool sub = gm->sub.count > 1;
    float *gc = (sub && grad_coords) ? ws.gtmp : grad_coords;
    float *gw = (sub && grad_weights) ? ws.wtmp : grad_weights;
    if (tables != Tables::kUseBuilt) {
        const int stop = timing_prep_stop();
        rc = hip_status(mg::launch_prep(gm->gs, bt, ws, stop, (hipStream_t)stream));
        if (rc != MG_OK || stop != 0) return rc;    // a prep kernel cut short leaves no tables to read
    }
    const unsigned expect = tables == Tables::kUseBuilt ? mg::workspace_tag(gm->gs, bt) : 0u;
    rc = hip_status(mg::launch_backward(gm->gs, bt, ws, grad_out, grad_is_double, gc, gw, expect,
                                        take_events(), (hipStream_t)stream));
    if (rc != MG_OK || !sub) return rc;
    if (grad_coords)
        rc = hip_status(mg::launch_sum_subgrids(gm->sub.count, B, (size_t)N * 3, gc, grad_coords,
                                                (hipStream_t)stream));
    if (rc == MG_OK && grad_weights)
        rc = hip_status(mg::launch_sum_subgrids(gm->sub.count, B, (size_t)N * T, gw, grad_weights,
                                                (hipStream_t)stream));
    return rc;
}

int mg_backward_index(const mg_gridmaker *gm, int B, int N, int T, const float *coords,
                      const int32_t *types, const float *radii, const int32_t *natoms,
                      const float *centers, const float *quats, const float *translations,
                      const float *grad_out, float *grad_coords, void *workspace,
                      size_t workspace_bytes, void *stream)
{
    if (!types) return MG_ENULL;
    return backward_call(gm, B, N, T, coords, types, nullptr, radii, natoms, centers, quats,
                         translations, grad_out, false, grad_coords, nullptr, workspace,
                         workspace_bytes, stream);
}

int mg_backward_index_prepared(const mg_gridmaker *gm, int B, int N, int T,
                               const float *grad_out, float *grad_coords, void *workspace,
                               size_t workspace_bytes, void *stream)
{
    return backward_call(gm, B, N, T, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr,
                         nullptr, grad_out, false, grad_coords, nullptr, workspace, workspace_bytes,
                         stream, Tables::kUseBuilt, true);
}

int mg_backward_vector_prepared(const mg_gridmaker *gm, int B, int N, int T, const float *weights,
                                const float *radii, const float *grad_out, float *grad_coords,
                                float *grad_weights, void *workspace, size_t workspace_bytes,
                                void *stream)
{
    if (!weights) return MG_ENULL;
    return backward_call(gm, B, N, T, nullptr, nullptr, weights, radii, nullptr, nullptr, nullptr,
                         nullptr, grad_out, false, grad_coords, grad_weights, workspace,
                         workspace_bytes, stream, Tables::kUseBuilt);
}

int mg_backward_index_f64(const mg_gridmaker *gm, int B, int N, int T, const float *coords,
                          const int32_t *types, const float *radii, const int32_t *natoms,
                          const float *centers, const float *quats, const float *translations,
                          const double *grad_out, float *grad_coords, void *workspace,
                          size_t workspace_bytes, void *stream)
{
    if (!types) return MG_ENULL;
    return backward_call(gm, B, N, T, coords, types, nullptr, radii, natoms, centers, quats,
                         translations, grad_out, true, grad_coords, nullptr, workspace,
                         workspace_bytes, stream);
}

int mg_backward_vector(const mg_gridmaker *gm, int B, int N, int T, const float *coords,
                       const float *weights, const float *radii, const int32_t *natoms,
                       const float *centers, const float *quats, const float *translations,
                       const float *grad_out, float *grad_coords, float *grad_weights,
                       void *workspace, size_t workspace_bytes, void *stream)
{
    if (!weights) return MG_ENULL;
    return backward_call(gm, B, N, T, coords, nullptr, weights, radii, natoms, centers, quats,
                         translations, grad_out, false, grad_coords, grad_weights, workspace,
                         workspace_bytes, stream);
}

int mg_backward_vector_f64(const mg_gridmaker *gm, int B, int N, int T, const float *coords,
                           const float *weights, const float *radii, const int32_t *natoms,
                           const float *centers, const float *quats, const float *translations,
                           const double *grad_out, float *grad_coords, float *grad_weights,
                           void *workspace, size_t workspace_bytes, void *stream)
{
    if (!weights) return MG_ENULL;
    return backward_call(gm, B, N, T, coords, nullptr, weights, radii, natoms, centers, quats,
                         translations, grad_out, true, grad_coords, grad_weights, workspace,
                         workspace_bytes, stream);
}

const char *mg_strerror(int code)
{
    switch (code) {
    case MG_OK: return "ok";
    case MG_ENULL: return "a required pointer is NULL";
    case MG_ESHAPE: return "bad shape: B, N, T must be >= 1, B <= 65535, 1 <= D <= 1024, sizes must fit";
    case MG_EPARAM: return "bad parameter: resolution, radius_scale and gaussian_radius_multiple must be finite and positive";
    case MG_EWORKSPACE: return "workspace is NULL, not 32-byte aligned, or smaller than mg_workspace_bytes";
    case MG_EHIP: return "the HIP runtime refused a launch (mg_last_hip_error has the hipError_t)";
    case MG_EMODE: return "call not defined for this GridMaker (binary backward, or vector types without radius_type_indexed)";
    case MG_EALIGN: return "an array argument is not 4-byte aligned";
    case MG_ENOMEM: return "out of host memory";
    default: return "unknown error code";
    }
}

int mg_last_hip_error(void) { return g_last_hip_error; }

int mg_time_next_kernel(void *start_event, void *stop_event)
{
    g_ev_start = (hipEvent_t)start_event;
    g_ev_stop = (hipEvent_t)stop_event;
    return MG_OK;
}

int mg_set_option(const char *key, int value)
{
    if (!key) return MG_ENULL;
    if (std::strcmp(key, "tile_floats") == 0) {
        if (value != 0 && value != 512 && value != 1024 && value != 2048 && value != 4096) return MG_EPARAM;
        g_tile_floats = value;
        return MG_OK;
    }
    if (std::strcmp(key, "waves_per_tile") == 0) {
        if (value != 0 && value != 1 && value != 2 && value != 4) return MG_EPARAM;
        g_waves_per_tile = value;
        return MG_OK;
    }
    if (std::strcmp(key, "xcd_run") == 0) {
        if (value < 0 || value > 32768 || (value & (value - 1)) != 0) return MG_EPARAM;
        g_xcd_run = value;
        return MG_OK;
    }
    if (std::strcmp(key, "keep_alive") == 0) {
        if (value != 0 && value != 1 && value != 64 && value != 128 && value != 256 && value != 512 &&
            value != 1024)
            return MG_EPARAM;
        g_keep_alive = value;
        return MG_OK;
    }
    if (std::strcmp(key, "keep_alive_stride") == 0) {
        if (value != 1 && value != 2 && value != 4 && value != 8) return MG_EPARAM;
        g_keep_alive_stride = value;
        return MG_OK;
    }
    if (std::strcmp(key, "single_launch") == 0) {
        if (value != 0 && value != 1) return MG_EPARAM;
        g_single_launch = value;
        return MG_OK;
    }
    if (std::strcmp(key, "tile_order") == 0) {
        if (value != 0 && value != 1) return MG_EPARAM;
        g_tile_order = value;
        return MG_OK;
    }
    if (std::strcmp(key, "lds_floor") == 0) {
        if (value < -1 || value > 65536) return MG_EPARAM;
        g_lds_floor = value;
        return MG_OK;
    }
#ifdef MG_TIMING_AIDS
    if (std::strcmp(key, "prep_stop") == 0) {
        if (value < 0 || value > 6) return MG_EPARAM;
        g_prep_stop = value;
        return MG_OK;
    }
    if (std::strcmp(key, "debug") == 0) {
        if (value < 0 || value > 3) return MG_EPARAM;
        g_debug = value;
        return MG_OK;
    }
#endif
    return MG_EPARAM;
}

}  // extern "C"
