// C ABI of libxconv: argument validation, scratch layout, kernel sequencing and
// the optional per-kernel event timing.  Declarations and their contracts are
// in include/xconv.h.
#include <cstdlib>
#include <cstring>
#include <mutex>
#include <vector>

extern char **environ;

#include "common.h"
#include "launch.h"

using namespace xc;

namespace {

inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }
inline bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
inline size_t elem_bytes(int dtype) { return dtype == XCONV_F32 ? 4 : 2; }
inline int out_extent(int in, int k, int stride, int pad)
{
    const int span = in + 2 * pad - k;
    return span < 0 ? 0 : span / stride + 1;
}

// ---- event timing ----------------------------------------------------------
struct ProfRec {
    int id;
    hipEvent_t a, b;
};
bool g_prof_on = false;
std::vector<ProfRec> g_prof;
std::mutex g_prof_mu;

struct ProfScope {
    hipStream_t st;
    int slot = -1;
    ProfScope(int id, hipStream_t s) : st(s)
    {
        if (!g_prof_on) return;
        ProfRec r{id, nullptr, nullptr};
        if (hipEventCreate(&r.a) != hipSuccess || hipEventCreate(&r.b) != hipSuccess) return;
        (void)hipEventRecord(r.a, st);
        std::lock_guard<std::mutex> lk(g_prof_mu);
        g_prof.push_back(r);
        slot = (int)g_prof.size() - 1;
    }
    ~ProfScope()
    {
        if (slot < 0) return;
        std::lock_guard<std::mutex> lk(g_prof_mu);
        (void)hipEventRecord(g_prof[slot].b, st);
    }
};

#define XC_LAUNCH(id, st, expr)               \
    do {                                      \
        ProfScope _ps((id), (st));            \
        hipError_t _e = (expr);               \
        if (_e != hipSuccess) return XCONV_EHIP; \
    } while (0)

// ---- plans -------------------------------------------------------------------
struct PlanKey {
    int v[14];
    bool operator==(const PlanKey &o) const
    {
        for (int i = 0; i < 14; ++i)
            if (v[i] != o.v[i]) return false;
        return true;
    }
};
struct PlanEntry {
    PlanKey key;
    CorrParams P;   // launch plan of corr_kernel; with `ws` only the fields the reduction and expansion read
    WsParams Wp;    // launch plan of corr_ws_kernel (ws == 1, 16-bit storage), corr_ws32_kernel (ws == 2, fp32) or corr_row_kernel (ws == 3)
    int ws;
    bool ok;
};
std::mutex g_plan_mu;
std::vector<PlanEntry> g_plans;

// The plan functions read XCONV_* overrides from the environment, so the overrides in force are part of
// the cache key: a plan made under one setting is never handed out under another.
int plan_override_hash()
{
    uint32_t h = 2166136261u;
    for (char **e = environ; e && *e; ++e) {
        if (strncmp(*e, "XCONV_", 6) != 0) continue;
        for (const char *c = *e; *c; ++c) h = (h ^ (uint8_t)*c) * 16777619u;
        h = (h ^ 0xffu) * 16777619u;
    }
    return (int)h;
}

// allow_row: the row-sweep kernel may be chosen (2-D layers; the volumetric entry points, which hand the kernels
// depth slices through an offset table, keep to the kernels that know that table)
bool get_plan(PlanEntry &out, int dtype, int B, int C_out, int H, int W, int kH, int kW, int sh, int sw, int ph, int pw, int CS,
              bool dy_aligned, bool allow_row = true)
{
    PlanKey k{{dtype, B, C_out, H, W, kH, kW, sh, sw, ph, pw, CS, (dy_aligned ? 1 : 0) | (allow_row ? 2 : 0), plan_override_hash()}};
    {
        std::lock_guard<std::mutex> lk(g_plan_mu);
        for (const PlanEntry &e : g_plans)
            if (e.key == k) {
                out = e;
                return e.ok;
            }
    }
    PlanEntry e;
    e.key = k;
    e.P = CorrParams{};
    e.Wp = WsParams{};
    // the producer/consumer kernel reads dY in place, so the caller's planes must be usable as they are
    e.ws = (dy_aligned && allow_row && plan_corr_row(e.Wp, dtype, B, C_out, H, W, kH, kW, sh, sw, ph, pw, CS)) ? 3 : 0;
    if (!e.ws && dy_aligned && plan_corr_ws(e.Wp, dtype, B, C_out, H, W, kH, kW, sh, sw, ph, pw, CS)) e.ws = 1;
    if (!e.ws && dy_aligned && plan_corr_ws32(e.Wp, dtype, B, C_out, H, W, kH, kW, sh, sw, ph, pw, CS)) e.ws = 2;
    if (e.ws) {
        e.ok = true;
        e.P.C_out = C_out;
        e.P.S = e.Wp.S; e.P.NS = e.Wp.NS;
        e.P.K2 = e.Wp.K2; e.P.JP = e.Wp.JP; e.P.MP = e.Wp.MP;
        e.P.Ho = e.Wp.Ho; e.P.Wo = e.Wp.Wo;
    } else {
        e.ok = plan_corr(e.P, dtype, B, C_out, H, W, kH, kW, sh, sw, ph, pw, CS, dy_aligned);
    }
    out = e;
    std::lock_guard<std::mutex> lk(g_plan_mu);
    if (g_plans.size() >= 64) g_plans.erase(g_plans.begin());
    g_plans.push_back(e);
    return e.ok;
}

hipError_t launch_ws_plan(int dtype, const PlanEntry &E, hipStream_t st)
{
    if (E.ws == 3) return launch_corr_row(dtype, E.Wp, st);
    return E.ws == 2 ? launch_corr_ws32(E.Wp, st) : launch_corr_ws(dtype, E.Wp, st);
}

// distribution and keep probability in the form the generator takes
int probe_code(const xconv_desc *d) { return d->probe | (d->keep_q15 << 8); }

size_t z_bytes(const xconv_desc *d) { return align_up((size_t)d->C_in * d->r * sizeof(float), 256); }
// Z in the fragment order of the probe kernels, behind the fp32 Z in the probe workspace
size_t zfrag_bytes(const xconv_desc *d)
{
    return align_up(zpack_bytes(d->dtype, d->C_in, d->r, d->probe == XCONV_RADEMACHER), 256);
}

// dY planes that are not a whole number of 16-byte vectors are repacked into scratch
int dy_pitch(const xconv_desc *d)
{
    const int n = out_extent(d->H, d->kH, d->stride_h, d->pad_h) * out_extent(d->W, d->kW, d->stride_w, d->pad_w);
    return round_up(n, d->dtype == XCONV_F32 ? 4 : 8);
}
size_t dy_repack_bytes(const xconv_desc *d)
{
    const int n = out_extent(d->H, d->kH, d->stride_h, d->pad_h) * out_extent(d->W, d->kW, d->stride_w, d->pad_w);
    // a channels-last dY is always brought into plane form first
    if (dy_pitch(d) == n && d->layout == XCONV_NCHW) return 0;
    return align_up((size_t)d->B * d->C_out * dy_pitch(d) * elem_bytes(d->dtype), 256);
}

}  // namespace

extern "C" {

xconv_status xconv_check_desc(const xconv_desc *d)
{
    if (!d) return XCONV_EINVAL;
    if (d->B < 1 || d->C_in < 1 || d->C_out < 1 || d->H < 1 || d->W < 1) return XCONV_EINVAL;
    if (d->kH < 1 || d->kW < 1 || d->stride_h < 1 || d->stride_w < 1 || d->pad_h < 0 || d->pad_w < 0) return XCONV_EINVAL;
    if (d->r < 1 || d->keep_q15 < 0 || d->keep_q15 > 32767) return XCONV_EINVAL;
    if (d->dtype < XCONV_F32 || d->dtype > XCONV_F16) return XCONV_EINVAL;
    if (d->layout < XCONV_NCHW || d->layout > XCONV_NHWC) return XCONV_EINVAL;
    if (d->probe < XCONV_RADEMACHER || d->probe > XCONV_USER_Z) return XCONV_EINVAL;
    if (out_extent(d->H, d->kH, d->stride_h, d->pad_h) < 1 || out_extent(d->W, d->kW, d->stride_w, d->pad_w) < 1) return XCONV_EINVAL;
    if (d->r > 1024 || d->C_in > 65536 || d->C_out > 65536 || (long long)d->kH * d->kW > 49) return XCONV_EUNSUPPORTED;
    if ((long long)d->H * d->W > 0x7fffffffLL / 8 || (long long)(d->H + 2 * d->pad_h) * (d->W + 2 * d->pad_w) > 0x7fffffffLL / 8)
        return XCONV_EUNSUPPORTED;
    if (d->pad_h > 4096 || d->pad_w > 4096 || d->stride_h > 4096 || d->stride_w > 4096) return XCONV_EUNSUPPORTED;
    return XCONV_OK;
}

size_t xconv_xt_bytes(const xconv_desc *d)
{
    if (xconv_check_desc(d) != XCONV_OK) return 0;
    return (size_t)d->B * d->H * d->W * round_up(d->r, 16) * elem_bytes(d->dtype);
}

size_t xconv_workspace_bytes(const xconv_desc *d, int op)
{
    if (xconv_check_desc(d) != XCONV_OK) return 0;
    if (op == XCONV_OP_PROBE) return z_bytes(d) + zfrag_bytes(d);
    PlanEntry E;
    if (op == XCONV_OP_ESTIMATE) {
        if (!get_plan(E, d->dtype, d->B, d->C_out, d->H, d->W, d->kH, d->kW, d->stride_h, d->stride_w, d->pad_h, d->pad_w,
                      round_up(d->r, 16), true))
            return 0;
        return z_bytes(d) + align_up(corr_partial_bytes(E.P), 256) + dy_repack_bytes(d);
    }
    if (op == XCONV_OP_EXACT) {
        const int CSx = round_up(d->C_in, 16);
        if (!get_plan(E, d->dtype, d->B, d->C_out, d->H, d->W, d->kH, d->kW, d->stride_h, d->stride_w, d->pad_h, d->pad_w, CSx, true))
            return 0;
        return align_up((size_t)d->B * d->H * d->W * CSx * elem_bytes(d->dtype), 256) + align_up(corr_partial_bytes(E.P), 256) + dy_repack_bytes(d);
    }
    return 0;
}

xconv_status xconv_probe_matrix(const xconv_desc *d, float *Z_host)
{
    xconv_status s = xconv_check_desc(d);
    if (s != XCONV_OK) return s;
    if (!Z_host || d->probe == XCONV_USER_Z) return XCONV_EINVAL;
    host_probe_matrix(probe_code(d), d->seed, d->C_in * d->r, Z_host);
    return XCONV_OK;
}

xconv_status xconv_probe_matrix_dev(const xconv_desc *d, float *Z_dev, void *stream)
{
    xconv_status s = xconv_check_desc(d);
    if (s != XCONV_OK) return s;
    if (!Z_dev || d->probe == XCONV_USER_Z) return XCONV_EINVAL;
    hipStream_t st = static_cast<hipStream_t>(stream);
    XC_LAUNCH(K_GEN_Z, st, launch_gen_z(Z_dev, d->C_in * d->r, probe_code(d), d->seed, st));
    return XCONV_OK;
}

}  // extern "C"

namespace {

// Forward probe over B images of HW pixels each; `sm` says where the output goes in Xt
// (SliceMap{} for 2-D layers: plain order).  `HWv`: extent whose divisibility decides the vector loads.
// zmul: factor on a given Z, applied where Z is brought into fragment order (callers that pass one check
// probe_scales_z first)
bool probe_scales_z(const xconv_desc *d, int HWv, const void *X_dev, const void *ws_dev)
{
    return ws_dev && probe_fast_path_ok(d->dtype, d->C_in, HWv, d->layout == XCONV_NHWC) && aligned16(X_dev);
}

xconv_status probe_impl(const xconv_desc *d, int HW, int HWv, SliceMap sm, const void *X_dev, void *Xt_dev, const float *Z_dev,
                        void *ws_dev, size_t ws_bytes, hipStream_t st, float zmul = 1.0f)
{
    if (!X_dev || !Xt_dev) return XCONV_EINVAL;
    if (!aligned16(Xt_dev) || (reinterpret_cast<uintptr_t>(X_dev) & (elem_bytes(d->dtype) - 1)) != 0) return XCONV_EINVAL;
    const int CS = round_up(d->r, 16);
    const bool z_exact16 = d->probe == XCONV_RADEMACHER;
    const bool nhwc = d->layout == XCONV_NHWC;
    const bool fast = probe_fast_path_ok(d->dtype, d->C_in, HWv, nhwc) && aligned16(X_dev);
    const size_t zb = z_bytes(d), fb = zfrag_bytes(d);
    if (!Z_dev && d->probe == XCONV_USER_Z) return XCONV_EINVAL;
    if (ws_dev) {
        if (!aligned16(ws_dev)) return XCONV_EINVAL;
        if (ws_bytes < zb + fb) return XCONV_EWORKSPACE;
    } else if (!Z_dev) {
        return XCONV_EINVAL;
    }
    if (zmul != 1.0f && !(Z_dev && probe_scales_z(d, HWv, X_dev, ws_dev))) return XCONV_EINVAL;
    if (fast) {
        // With scratch, Z goes to the kernels in fragment order (drawn from the seed when no Z
        // is given); without it, every workgroup gathers its fragments from Z_dev.
        void *zpack = ws_dev ? static_cast<char *>(ws_dev) + zb : nullptr;
        // a small +-1 matrix defined by the seed is cheaper to draw in every workgroup than in a launch of its own
        {
            const char *v = getenv("XCONV_PROBE_DRAW");   // sweeps: largest Z drawn inside the probe kernel, Rademacher / Gaussian
            const long long lim_r = v ? atoll(v) : 1024, lim_g = v ? atoll(v) : 0;
            if (!Z_dev && (long long)d->C_in * d->r <= (d->probe == XCONV_RADEMACHER ? lim_r : lim_g)) zpack = nullptr;
            // 16-bit storage: a dense +-1 matrix of any size the kernel's word table holds
            if (!Z_dev && !v && d->dtype != XCONV_F32 && probe_draws_words(d->C_in, d->r, probe_code(d))) zpack = nullptr;
        }
        if (zpack) XC_LAUNCH(K_PACK_Z, st, launch_pack_z(d->dtype, Z_dev, zpack, d->C_in, d->r, z_exact16, probe_code(d), d->seed, nhwc, st, zmul));
        XC_LAUNCH(K_PROBE, st, launch_probe(d->dtype, X_dev, Z_dev, zpack, Xt_dev, d->B, d->C_in, HW, d->r, CS, z_exact16, nhwc, sm,
                                            probe_code(d), d->seed, st));
    } else {
        const float *Z = Z_dev;
        if (!Z) {
            float *zw = static_cast<float *>(ws_dev);
            XC_LAUNCH(K_GEN_Z, st, launch_gen_z(zw, d->C_in * d->r, probe_code(d), d->seed, st));
            Z = zw;
        }
        XC_LAUNCH(K_PROBE_GENERIC, st, launch_probe_generic(d->dtype, X_dev, Z, Xt_dev, d->B, d->C_in, HW, d->r, CS, nhwc, sm, st));
    }
    return XCONV_OK;
}

// ---- volumetric layers: geometry of the slice layout -------------------------------
struct Vol {
    int sd;              // depth stride
    int Do;              // output depth
    int period;          // slots per image in the slice-major buffers
    long long B2;        // images of the 2-D problem the kernels see: B * period depth slices
    long long run;       // slices per run of Xt: B2 and (kD-1)/sd zero slices behind the last image
    long long slices;    // slices of Xt: sd runs
    size_t slice_bytes;  // one depth slice of Xt
};
Vol vol_of(const xconv3d_desc *v)
{
    Vol g;
    g.sd = v->stride_d;
    g.Do = (v->D + 2 * v->pad_d - v->kD) / g.sd + 1;
    const int reach = g.Do + (v->kD - 1) / g.sd;   // slots a kernel-depth offset can pair an image's output slices with
    if (g.sd == 1) {
        // the pad_d leading slots of the next image are zero and take the overhang
        g.period = v->D + v->pad_d;
    } else {
        const int used = (v->D - 1 + v->pad_d) / g.sd + 1;
        g.period = used > reach ? used : reach;
    }
    g.B2 = (long long)v->l.B * g.period;
    g.run = g.B2 + (v->kD - 1) / g.sd;   // the deepest offset reads that far past the last slot (against zero slots of dY)
    g.slices = (long long)g.sd * g.run;
    g.slice_bytes = (size_t)v->l.H * v->l.W * round_up(v->l.r, 16) * elem_bytes(v->l.dtype);
    return g;
}
SliceMap vol_map(const xconv3d_desc *v, const Vol &g)
{
    SliceMap sm;
    sm.HWs = v->l.H * v->l.W;
    sm.D = v->D;
    sm.pd = v->pad_d;
    sm.sd = g.sd;
    sm.period = g.period;
    sm.run = g.run;
    return sm;
}
// The producer/consumer kernels read the caller's dY [B, C_out, Do, H'*W'] in place (depth slots of volumes,
// WsParams::vol_*) when its byte offsets fit; otherwise dY is first copied into slice-major planes.
bool vol_dy_in_place(const xconv3d_desc *v, const Vol &g, PlanEntry &E, const void *dY_dev)
{
    const xconv_desc *d = &v->l;
    const char *force_copy = getenv("XCONV_VOL_COPY");   // tests: take the copy route also where in-place reads fit
    if (E.ws == 0 || d->layout != XCONV_NCHW || !aligned16(dY_dev) || (force_copy && *force_copy == '1')) return false;
    const long long bytes = (long long)d->B * d->C_out * g.Do * E.P.Ho * E.P.Wo * (long long)elem_bytes(d->dtype);
    if (bytes > (1LL << 30) || g.B2 >= (1LL << 22)) return false;
    E.Wp.vol_period = g.period;
    E.Wp.vol_Do = g.Do;
    E.Wp.vol_bytes = (uint32_t)bytes;
    return true;
}

// scratch of the correlations of a volumetric layer: kD sets of S partial tiles, then the kD reduced tiles
size_t vol_tile_bytes(const CorrParams &P) { return (size_t)P.K2 * P.JP * P.MP * sizeof(float); }
size_t vol_partial_bytes(const CorrParams &P, int kD) { return align_up((size_t)kD * P.S * vol_tile_bytes(P), 256); }
// first slice of Xt (or of X in slice form) that kernel-depth offset kz pairs with slice 0 of dY
size_t vol_offset_slices(const Vol &g, int kz) { return (size_t)(kz % g.sd) * (size_t)g.run + (size_t)(kz / g.sd); }
// plane pitch of the slice-major copy of dY for the kernel the plan selects
int vol_dy_pitch(const xconv3d_desc *v, const PlanEntry &E)
{
    const int n = E.P.Ho * E.P.Wo;
    return E.ws ? n : round_up(n, v->l.dtype == XCONV_F32 ? 4 : 8);
}
// CS: channel stride of the slices the correlation reads (r or, on the exact path, C_in, rounded up to 16)
bool vol_plan(PlanEntry &E, const xconv3d_desc *v, int CS)
{
    const xconv_desc *d = &v->l;
    const Vol g = vol_of(v);
    if (g.B2 > 0x7fffffffLL) return false;
    return get_plan(E, d->dtype, (int)g.B2, d->C_out, d->H, d->W, d->kH, d->kW, d->stride_h, d->stride_w, d->pad_h, d->pad_w, CS, true, false);
}

}  // namespace

extern "C" {

xconv_status xconv_probe_fwd(const xconv_desc *d, const void *X_dev, void *Xt_dev, const float *Z_dev, void *ws_dev,
                             size_t ws_bytes, void *stream)
{
    xconv_status s = xconv_check_desc(d);
    if (s != XCONV_OK) return s;
    return probe_impl(d, d->H * d->W, d->H * d->W, SliceMap{}, X_dev, Xt_dev, Z_dev, ws_dev, ws_bytes, static_cast<hipStream_t>(stream));
}

xconv_status xconv_dw_estimate(const xconv_desc *d, const void *dY_dev, const void *Xt_dev, const float *Z_dev, float *dW_dev,
                               void *ws_dev, size_t ws_bytes, void *stream)
{
    xconv_status s = xconv_check_desc(d);
    if (s != XCONV_OK) return s;
    if (!dY_dev || !Xt_dev || !dW_dev || !ws_dev) return XCONV_EINVAL;
    if (!aligned16(Xt_dev) || !aligned16(ws_dev) || (reinterpret_cast<uintptr_t>(dW_dev) & 3u) != 0) return XCONV_EINVAL;
    if (!aligned16(dY_dev)) return XCONV_EINVAL;
    if (!Z_dev && d->probe == XCONV_USER_Z) return XCONV_EINVAL;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const int CS = round_up(d->r, 16);
    PlanEntry E;
    if (!get_plan(E, d->dtype, d->B, d->C_out, d->H, d->W, d->kH, d->kW, d->stride_h, d->stride_w, d->pad_h, d->pad_w, CS,
                  aligned16(dY_dev)))
        return XCONV_EUNSUPPORTED;
    CorrParams &P = E.P;
    const size_t zb = z_bytes(d), pb = align_up(corr_partial_bytes(P), 256), rb = dy_repack_bytes(d);
    if (ws_bytes < zb + pb + rb) return XCONV_EWORKSPACE;
    // Z[s] is only needed by the expansion: it is redrawn by spare workgroups of the reduction launch
    const float *Z = Z_dev;
    float *zw = nullptr;
    if (!Z) {
        zw = static_cast<float *>(ws_dev);
        Z = zw;
    }
    P.dY = dY_dev;
    if (d->layout == XCONV_NHWC) {
        // channels-last dY -> the plane form the kernels read (pitch of the kernel that runs)
        void *packed = static_cast<char *>(ws_dev) + zb + pb;
        XC_LAUNCH(K_REPACK, st, launch_to_nchw(d->dtype, dY_dev, packed, d->B, d->C_out, P.Ho * P.Wo, E.ws ? P.Ho * P.Wo : dy_pitch(d), st));
        P.dY = packed;
    } else if (rb && !E.ws) {
        void *packed = static_cast<char *>(ws_dev) + zb + pb;
        XC_LAUNCH(K_REPACK, st, launch_repack_planes(d->dtype, dY_dev, packed, (long long)d->B * d->C_out, P.Ho * P.Wo, dy_pitch(d), st));
        P.dY = packed;
    }
    P.A = Xt_dev;
    P.part = reinterpret_cast<float *>(static_cast<char *>(ws_dev) + zb);
    // one launch for the second pass: Z[s], if it has to be redrawn, is drawn by the workgroups of the correlation launch
    const bool fused = reduce_expand_fused(P, Z_dev != nullptr, false, d->C_in, d->r, probe_code(d));
    if (fused && zw) {
        P.zout = E.Wp.zout = zw;
        P.nz = E.Wp.nz = d->C_in * d->r;
        P.zdist = E.Wp.zdist = probe_code(d);
        P.zseed = E.Wp.zseed = d->seed;
    }
    if (E.ws) {
        E.Wp.dY = P.dY;
        E.Wp.A = Xt_dev;
        E.Wp.part = P.part;
        XC_LAUNCH(K_CORR, st, launch_ws_plan(d->dtype, E, st));
    } else {
        XC_LAUNCH(K_CORR, st, launch_corr(d->dtype, P, st));
    }
    if (fused) {
        XC_LAUNCH(K_PASS2, st, launch_reduce_expand(P, Z, false, dW_dev, d->C_in, d->r, d->keep_q15 != 0, probe_code(d), d->seed, 1, st));
        return XCONV_OK;
    }
    XC_LAUNCH(K_REDUCE, st, launch_reduce(P, st, zw, d->C_in * d->r, probe_code(d), d->seed));
    XC_LAUNCH(K_EXPAND, st, launch_expand(P, Z, dW_dev, d->C_in, d->r, st, d->keep_q15 != 0));
    return XCONV_OK;
}

}  // extern "C"

// ---- the estimate without a workspace argument --------------------------------------------------
// Scratch of xconv_dw_estimate_static: a device array of the library itself, one copy per GPU, alive until the
// process ends.  Its name is a host-side stand-in here; the address on a device comes from hipGetSymbolAddress,
// asked for once per device with that device current, and only that address is ever handed to a kernel.
static __device__ __align__(256) unsigned char scratch[XCONV_STATIC_SCRATCH_BYTES];

namespace {

constexpr int kMaxDevices = 64;
std::mutex g_scratch_mu;
void *g_scratch_ptr[kMaxDevices] = {};

// address of `scratch` on the current device (nullptr: the runtime would not say)
void *static_scratch()
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return nullptr;
    std::lock_guard<std::mutex> lk(g_scratch_mu);
    if (!g_scratch_ptr[dev]) {
        void *ptr = nullptr;
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess) return nullptr;
        g_scratch_ptr[dev] = ptr;
    }
    return g_scratch_ptr[dev];
}

}  // namespace

extern "C" {

size_t xconv_static_scratch_bytes(void) { return XCONV_STATIC_SCRATCH_BYTES; }

xconv_status xconv_dw_estimate_static(const xconv_desc *d, const void *dY_dev, const void *Xt_dev, const float *Z_dev, float *dW_dev,
                                      void *stream)
{
    xconv_status s = xconv_check_desc(d);
    if (s != XCONV_OK) return s;
    const size_t need = xconv_workspace_bytes(d, XCONV_OP_ESTIMATE);
    if (need == 0) return XCONV_EUNSUPPORTED;
    if (need > (size_t)XCONV_STATIC_SCRATCH_BYTES) return XCONV_EWORKSPACE;
    void *ws = static_scratch();
    if (!ws) return XCONV_EHIP;
    // every partial sum the kernels read from the scratch is written earlier in the same call: nothing to clear
    return xconv_dw_estimate(d, dY_dev, Xt_dev, Z_dev, dW_dev, ws, XCONV_STATIC_SCRATCH_BYTES, stream);
}

}  // extern "C"

namespace {

// Exact-gradient path.  A_ready != nullptr: the activation is already channels-last [B, H, W, C_in rounded up
// to 16] with zero pad columns (X_dev is then ignored and may be null).
xconv_status exact_impl(const xconv_desc *d, const void *dY_dev, const void *X_dev, const void *A_ready, float *dW_dev, void *ws_dev,
                        size_t ws_bytes, void *stream)
{
    xconv_status s = xconv_check_desc(d);
    if (s != XCONV_OK) return s;
    if (A_ready) X_dev = A_ready;
    if (!dY_dev || !X_dev || !dW_dev || !ws_dev) return XCONV_EINVAL;
    if (!aligned16(ws_dev) || (reinterpret_cast<uintptr_t>(dW_dev) & 3u) != 0) return XCONV_EINVAL;
    const size_t eb = elem_bytes(d->dtype);
    if (!aligned16(dY_dev) || (reinterpret_cast<uintptr_t>(X_dev) & (eb - 1)) != 0) return XCONV_EINVAL;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const int CSx = round_up(d->C_in, 16), HW = d->H * d->W;
    PlanEntry E;
    if (!get_plan(E, d->dtype, d->B, d->C_out, d->H, d->W, d->kH, d->kW, d->stride_h, d->stride_w, d->pad_h, d->pad_w, CSx,
                  aligned16(dY_dev)))
        return XCONV_EUNSUPPORTED;
    CorrParams &P = E.P;
    const size_t xb = align_up((size_t)d->B * HW * CSx * eb, 256), pb = align_up(corr_partial_bytes(P), 256), rb = dy_repack_bytes(d);
    if (ws_bytes < xb + pb + rb) return XCONV_EWORKSPACE;
    // the correlation kernels read X channels-last with a channel stride that is a multiple of 16
    const void *A = ws_dev;
    if (A_ready) {
        A = A_ready;
    } else if (d->layout == XCONV_NCHW) {
        XC_LAUNCH(K_TO_NHWC, st, launch_to_nhwc(d->dtype, X_dev, ws_dev, d->B, d->C_in, HW, CSx, st));
    } else if (d->C_in == CSx && aligned16(X_dev)) {
        A = X_dev;  // already in that form
    } else {
        XC_LAUNCH(K_TO_NHWC, st, launch_pad_channels(d->dtype, X_dev, ws_dev, (long long)d->B * HW, d->C_in, CSx, st));
    }
    P.dY = dY_dev;
    if (d->layout == XCONV_NHWC) {
        void *packed = static_cast<char *>(ws_dev) + xb + pb;
        XC_LAUNCH(K_REPACK, st, launch_to_nchw(d->dtype, dY_dev, packed, d->B, d->C_out, P.Ho * P.Wo, E.ws ? P.Ho * P.Wo : dy_pitch(d), st));
        P.dY = packed;
    } else if (rb && !E.ws) {
        void *packed = static_cast<char *>(ws_dev) + xb + pb;
        XC_LAUNCH(K_REPACK, st, launch_repack_planes(d->dtype, dY_dev, packed, (long long)d->B * d->C_out, P.Ho * P.Wo, dy_pitch(d), st));
        P.dY = packed;
    }
    P.A = A;
    P.part = reinterpret_cast<float *>(static_cast<char *>(ws_dev) + xb);
    if (E.ws) {
        E.Wp.dY = P.dY;
        E.Wp.A = A;
        E.Wp.part = P.part;
        XC_LAUNCH(K_CORR, st, launch_ws_plan(d->dtype, E, st));
    } else {
        XC_LAUNCH(K_CORR, st, launch_corr(d->dtype, P, st));
    }
    if (reduce_expand_fused(P, false, true, d->C_in, d->r, 0)) {
        XC_LAUNCH(K_PASS2, st, launch_reduce_expand(P, nullptr, true, dW_dev, d->C_in, d->r, false, 0, 0, 1, st));
        return XCONV_OK;
    }
    XC_LAUNCH(K_REDUCE, st, launch_reduce(P, st));
    XC_LAUNCH(K_EXPAND, st, launch_expand(P, nullptr, dW_dev, d->C_in, d->r, st));
    return XCONV_OK;
}

}  // namespace

extern "C" {

xconv_status xconv_dw_exact(const xconv_desc *d, const void *dY_dev, const void *X_dev, float *dW_dev, void *ws_dev,
                            size_t ws_bytes, void *stream)
{
    return exact_impl(d, dY_dev, X_dev, nullptr, dW_dev, ws_dev, ws_bytes, stream);
}

// ---- forward convolution and exact input gradient (Sec. 2; Alg. 1 forward step 1) ----
static void conv_strides(int layout, int C, int H, int W, long long &sb, int &sc, int &sy, int &sx)
{
    if (layout == XCONV_NHWC) { sb = (long long)H * W * C; sc = 1; sy = W * C; sx = C; }
    else { sb = (long long)C * H * W; sc = H * W; sy = W; sx = 1; }
}

xconv_status xconv_conv_fwd(const xconv_desc *d, const void *X_dev, const void *W_dev, void *Y_dev, void *stream)
{
    xconv_status s = xconv_check_desc(d);
    if (s != XCONV_OK) return s;
    if (!X_dev || !W_dev || !Y_dev) return XCONV_EINVAL;
    const uintptr_t em = elem_bytes(d->dtype) - 1;
    if ((reinterpret_cast<uintptr_t>(X_dev) & em) || (reinterpret_cast<uintptr_t>(W_dev) & em) || (reinterpret_cast<uintptr_t>(Y_dev) & em)) return XCONV_EINVAL;
    const int Ho = out_extent(d->H, d->kH, d->stride_h, d->pad_h), Wo = out_extent(d->W, d->kW, d->stride_w, d->pad_w);
    if ((long long)d->C_in * d->H * d->W > 0x7fffffffLL || (long long)d->C_out * Ho * Wo > 0x7fffffffLL) return XCONV_EUNSUPPORTED;
    ConvGemmParams P{};
    P.in = X_dev; P.w = W_dev; P.out = Y_dev;
    P.Cin = d->C_in; P.Cout = d->C_out; P.Hi = d->H; P.Wi = d->W; P.Ho = Ho; P.Wo = Wo;
    P.kH = d->kH; P.kW = d->kW; P.sh = d->stride_h; P.sw = d->stride_w; P.ph = d->pad_h; P.pw = d->pad_w;
    P.transposed = 0;
    P.npix = (long long)d->B * Ho * Wo;
    conv_strides(d->layout, d->C_in, d->H, d->W, P.in_sb, P.in_sc, P.in_sy, P.in_sx);
    conv_strides(d->layout, d->C_out, Ho, Wo, P.out_sb, P.out_sc, P.out_sy, P.out_sx);
    P.w_sco = d->C_in * d->kH * d->kW;
    P.w_sci = d->kH * d->kW;
    hipStream_t st = static_cast<hipStream_t>(stream);
    XC_LAUNCH(K_CONV, st, launch_conv_gemm(d->dtype, P, st));
    return XCONV_OK;
}

xconv_status xconv_dx_exact(const xconv_desc *d, const void *dY_dev, const void *W_dev, void *dX_dev, void *stream)
{
    xconv_status s = xconv_check_desc(d);
    if (s != XCONV_OK) return s;
    if (!dY_dev || !W_dev || !dX_dev) return XCONV_EINVAL;
    const uintptr_t em = elem_bytes(d->dtype) - 1;
    if ((reinterpret_cast<uintptr_t>(dY_dev) & em) || (reinterpret_cast<uintptr_t>(W_dev) & em) || (reinterpret_cast<uintptr_t>(dX_dev) & em)) return XCONV_EINVAL;
    const int Ho = out_extent(d->H, d->kH, d->stride_h, d->pad_h), Wo = out_extent(d->W, d->kW, d->stride_w, d->pad_w);
    if ((long long)d->C_in * d->H * d->W > 0x7fffffffLL || (long long)d->C_out * Ho * Wo > 0x7fffffffLL) return XCONV_EUNSUPPORTED;
    ConvGemmParams P{};
    P.in = dY_dev; P.w = W_dev; P.out = dX_dev;
    P.Cin = d->C_out; P.Cout = d->C_in; P.Hi = Ho; P.Wi = Wo; P.Ho = d->H; P.Wo = d->W;
    P.kH = d->kH; P.kW = d->kW; P.sh = d->stride_h; P.sw = d->stride_w; P.ph = d->pad_h; P.pw = d->pad_w;
    P.transposed = 1;
    P.npix = (long long)d->B * d->H * d->W;
    conv_strides(d->layout, d->C_out, Ho, Wo, P.in_sb, P.in_sc, P.in_sy, P.in_sx);
    conv_strides(d->layout, d->C_in, d->H, d->W, P.out_sb, P.out_sc, P.out_sy, P.out_sx);
    P.w_sco = d->kH * d->kW;                 // the product's output channel is the layer's input channel n
    P.w_sci = d->C_in * d->kH * d->kW;       // and it contracts over the layer's output channels m
    hipStream_t st = static_cast<hipStream_t>(stream);
    XC_LAUNCH(K_CONV, st, launch_conv_gemm(d->dtype, P, st));
    return XCONV_OK;
}

xconv_status xconv_plan_info(const xconv_desc *d, int op, int32_t *out)
{
    xconv_status s = xconv_check_desc(d);
    if (s != XCONV_OK) return s;
    if (!out || (op != XCONV_OP_ESTIMATE && op != XCONV_OP_EXACT)) return XCONV_EINVAL;
    const int CS = round_up(op == XCONV_OP_ESTIMATE ? d->r : d->C_in, 16);
    PlanEntry E;
    if (!get_plan(E, d->dtype, d->B, d->C_out, d->H, d->W, d->kH, d->kW, d->stride_h, d->stride_w, d->pad_h, d->pad_w, CS, true))
        return XCONV_EUNSUPPORTED;
    if (E.ws) {
        const WsParams &Q = E.Wp;
        const int32_t v[16] = {Q.S, Q.NS, 1, Q.CW, Q.WM, Q.WJ, 1, Q.M_WG, Q.J_WG, (int32_t)(E.ws == 3 ? corr_row_lds_bytes(Q) : E.ws == 2 ? corr_ws32_lds_bytes(Q) : corr_ws_lds_bytes(Q)),
                               Q.NTM, Q.NTJ, Q.NOG, Q.CS, Q.NSUB, E.ws};
        for (int i = 0; i < 16; ++i) out[i] = v[i];
        return XCONV_OK;
    }
    const CorrParams &P = E.P;
    const int32_t v[16] = {P.S, P.NS, P.RB, P.CW, P.WM, P.WJ, P.WK, P.M_WG, P.J_WG, (int32_t)corr_lds_bytes(d->dtype, P),
                           P.NTM, P.NTJ, P.NOG, P.CS, P.NCHR, 0};
    for (int i = 0; i < 16; ++i) out[i] = v[i];
    return XCONV_OK;
}

xconv_status xconv_xt_unpack(const xconv_desc *d, const void *Xt_dev, float *out_dev, void *stream)
{
    xconv_status s = xconv_check_desc(d);
    if (s != XCONV_OK) return s;
    if (!Xt_dev || !out_dev) return XCONV_EINVAL;
    hipStream_t st = static_cast<hipStream_t>(stream);
    XC_LAUNCH(K_UNPACK, st, launch_unpack(d->dtype, Xt_dev, out_dev, d->B, d->H * d->W, d->r, round_up(d->r, 16), st));
    return XCONV_OK;
}

// ---- volumetric layers -----------------------------------------------------------
// Slice layout: the copy of dY holds `period` slots per image, output slice oz in slot oz, the
// rest zero.  Xt holds sd runs of the same slots; depth slice z of an image sits in slot
// (z + pd) / sd of run (z + pd) % sd, every other slot is zero.  Kernel-depth offset kz then
// pairs slot i of dY with slot i + kz / sd of run kz % sd of Xt for every i, and the partner is
// a zero slot whenever oz * sd + kz - pd leaves the image.

xconv_status xconv3d_check_desc(const xconv3d_desc *v)
{
    if (!v) return XCONV_EINVAL;
    xconv_status s = xconv_check_desc(&v->l);
    if (s != XCONV_OK) return s;
    if (v->D < 1 || v->kD < 1 || v->pad_d < 0 || v->stride_d < 1) return XCONV_EINVAL;
    if (v->D + 2 * v->pad_d - v->kD < 0) return XCONV_EINVAL;   // empty output
    if (v->kD > 7 || v->pad_d > v->kD - 1) return XCONV_EUNSUPPORTED;
    if ((long long)v->D * v->l.H * v->l.W > (1LL << 28)) return XCONV_EUNSUPPORTED;
    if (v->stride_d > 4096 || (long long)v->l.B * (v->D + 2 * v->pad_d) > 0x7fffffffLL) return XCONV_EUNSUPPORTED;
    return XCONV_OK;
}

size_t xconv3d_xt_bytes(const xconv3d_desc *v)
{
    if (xconv3d_check_desc(v) != XCONV_OK) return 0;
    const Vol g = vol_of(v);
    return (size_t)g.slices * g.slice_bytes;
}

size_t xconv3d_workspace_bytes(const xconv3d_desc *v, int op)
{
    if (xconv3d_check_desc(v) != XCONV_OK) return 0;
    const xconv_desc *d = &v->l;
    if (op == XCONV_OP_PROBE) return z_bytes(d) + zfrag_bytes(d);
    if (op != XCONV_OP_ESTIMATE && op != XCONV_OP_EXACT) return 0;
    const bool exact = op == XCONV_OP_EXACT;
    const int CS = round_up(exact ? d->C_in : d->r, 16);
    PlanEntry E;
    if (!vol_plan(E, v, CS)) return 0;
    const Vol g = vol_of(v);
    const size_t tile = (size_t)E.P.K2 * E.P.JP * E.P.MP * sizeof(float);
    // exact: channels-last slices of X in the layout of Xt take the place of Z
    const size_t head = exact ? align_up((size_t)g.slices * d->H * d->W * CS * elem_bytes(d->dtype), 256) : z_bytes(d);
    return head + vol_partial_bytes(E.P, v->kD) + align_up((size_t)v->kD * tile, 256) +
           align_up((size_t)g.B2 * d->C_out * vol_dy_pitch(v, E) * elem_bytes(d->dtype), 256);
}

xconv_status xconv3d_probe_fwd(const xconv3d_desc *v, const void *X_dev, void *Xt_dev, const float *Z_dev, void *ws_dev,
                               size_t ws_bytes, void *stream)
{
    xconv_status s = xconv3d_check_desc(v);
    if (s != XCONV_OK) return s;
    const xconv_desc *d = &v->l;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const int HW = d->H * d->W;
    const Vol g = vol_of(v);
    const SliceMap sm = vol_map(v, g);
    s = probe_impl(d, v->D * HW, HW, sm, X_dev, Xt_dev, Z_dev, ws_dev, ws_bytes, st);
    if (s != XCONV_OK) return s;
    XC_LAUNCH(K_ZERO_GAPS, st, launch_zero_gap_slices(Xt_dev, g.slice_bytes, d->B, sm, st));
    return XCONV_OK;
}

xconv_status xconv3d_dw_estimate(const xconv3d_desc *v, const void *dY_dev, const void *Xt_dev, const float *Z_dev, float *dW_dev,
                                 void *ws_dev, size_t ws_bytes, void *stream)
{
    xconv_status s = xconv3d_check_desc(v);
    if (s != XCONV_OK) return s;
    const xconv_desc *d = &v->l;
    if (!dY_dev || !Xt_dev || !dW_dev || !ws_dev) return XCONV_EINVAL;
    if (!aligned16(Xt_dev) || !aligned16(ws_dev) || (reinterpret_cast<uintptr_t>(dW_dev) & 3u) != 0) return XCONV_EINVAL;
    if ((reinterpret_cast<uintptr_t>(dY_dev) & (elem_bytes(d->dtype) - 1)) != 0) return XCONV_EINVAL;
    if (!Z_dev && d->probe == XCONV_USER_Z) return XCONV_EINVAL;
    hipStream_t st = static_cast<hipStream_t>(stream);
    PlanEntry E;
    if (!vol_plan(E, v, round_up(d->r, 16))) return XCONV_EUNSUPPORTED;
    CorrParams &P = E.P;
    const Vol g = vol_of(v);
    const int pitch = vol_dy_pitch(v, E);
    const size_t tile = (size_t)P.K2 * P.JP * P.MP * sizeof(float);
    const size_t zb = z_bytes(d), pb = vol_partial_bytes(P, v->kD), tb = align_up((size_t)v->kD * tile, 256);
    const size_t yb = align_up((size_t)g.B2 * d->C_out * pitch * elem_bytes(d->dtype), 256);
    if (ws_bytes < zb + pb + tb + yb) return XCONV_EWORKSPACE;
    char *ws = static_cast<char *>(ws_dev);
    const float *Z = Z_dev;
    float *zw = nullptr;
    if (!Z) {
        zw = reinterpret_cast<float *>(ws);
        Z = zw;
    }
    float *T3 = reinterpret_cast<float *>(ws + zb + pb);
    void *dy_slices = ws + zb + pb + tb;
    if (vol_dy_in_place(v, g, E, dY_dev)) {
        P.dY = dY_dev;
    } else {
        if (d->layout == XCONV_NHWC)
            XC_LAUNCH(K_REPACK, st, launch_dy_slices_nhwc(d->dtype, dY_dev, dy_slices, d->B, d->C_out, g.Do, g.period, P.Ho * P.Wo, pitch, st));
        else
            XC_LAUNCH(K_REPACK, st, launch_dy_slices(d->dtype, dY_dev, dy_slices, d->B, d->C_out, g.Do, g.period, P.Ho * P.Wo, pitch, st));
        P.dY = dy_slices;
    }
    float *part0 = reinterpret_cast<float *>(ws + zb);
    const bool fused = reduce_expand_fused(P, Z_dev != nullptr, false, d->C_in, d->r, probe_code(d), v->kD);
    for (int kz = 0; kz < v->kD; ++kz) {
        // (the first correlation launch also redraws Z[s] for the fused second pass)
        P.zout = E.Wp.zout = (fused && zw && kz == 0) ? zw : nullptr;
        P.nz = E.Wp.nz = d->C_in * d->r;
        P.zdist = E.Wp.zdist = probe_code(d);
        P.zseed = E.Wp.zseed = d->seed;
        const void *A = static_cast<const char *>(Xt_dev) + vol_offset_slices(g, kz) * g.slice_bytes;
        P.A = A;
        P.part = part0 + (size_t)kz * P.S * (tile / sizeof(float));
        if (E.ws) {
            E.Wp.dY = P.dY;
            E.Wp.A = A;
            E.Wp.part = P.part;
            XC_LAUNCH(K_CORR, st, launch_ws_plan(d->dtype, E, st));
        } else {
            XC_LAUNCH(K_CORR, st, launch_corr(d->dtype, P, st));
        }
    }
    // one reduction for all kernel-depth offsets; its spare workgroups redraw Z[s] for the expansion
    P.part = part0;
    if (fused) {
        XC_LAUNCH(K_PASS2, st, launch_reduce_expand(P, Z, false, dW_dev, d->C_in, d->r, d->keep_q15 != 0, probe_code(d), d->seed, v->kD, st));
        return XCONV_OK;
    }
    XC_LAUNCH(K_REDUCE, st, launch_reduce(P, st, zw, d->C_in * d->r, probe_code(d), d->seed, T3, v->kD));
    XC_LAUNCH(K_EXPAND, st, launch_expand(P, Z, dW_dev, d->C_in, d->r, st, d->keep_q15 != 0, T3, v->kD * P.K2));
    return XCONV_OK;
}

xconv_status xconv3d_dw_exact(const xconv3d_desc *v, const void *dY_dev, const void *X_dev, float *dW_dev, void *ws_dev,
                              size_t ws_bytes, void *stream)
{
    xconv_status s = xconv3d_check_desc(v);
    if (s != XCONV_OK) return s;
    const xconv_desc *d = &v->l;
    if (!dY_dev || !X_dev || !dW_dev || !ws_dev) return XCONV_EINVAL;
    if (!aligned16(ws_dev) || (reinterpret_cast<uintptr_t>(dW_dev) & 3u) != 0) return XCONV_EINVAL;
    const size_t eb = elem_bytes(d->dtype);
    if ((reinterpret_cast<uintptr_t>(dY_dev) & (eb - 1)) != 0 || (reinterpret_cast<uintptr_t>(X_dev) & (eb - 1)) != 0) return XCONV_EINVAL;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const int CSx = round_up(d->C_in, 16), HW = d->H * d->W;
    PlanEntry E;
    if (!vol_plan(E, v, CSx)) return XCONV_EUNSUPPORTED;
    CorrParams &P = E.P;
    const Vol g = vol_of(v);
    const int pitch = vol_dy_pitch(v, E);
    const size_t xslice = (size_t)HW * CSx * eb;
    const size_t tile = (size_t)P.K2 * P.JP * P.MP * sizeof(float);
    const size_t xb = align_up((size_t)g.slices * xslice, 256), pb = vol_partial_bytes(P, v->kD);
    const size_t tb = align_up((size_t)v->kD * tile, 256), yb = align_up((size_t)g.B2 * d->C_out * pitch * eb, 256);
    if (ws_bytes < xb + pb + tb + yb) return XCONV_EWORKSPACE;
    char *ws = static_cast<char *>(ws_dev);
    // X -> channels-last depth slices in the slice layout of Xt, zero slots between
    const SliceMap sm = vol_map(v, g);
    if (d->layout == XCONV_NHWC)
        XC_LAUNCH(K_TO_NHWC, st, launch_x_slices_nhwc(d->dtype, X_dev, ws, d->B, d->C_in, CSx, sm, st));
    else
        XC_LAUNCH(K_TO_NHWC, st, launch_to_slices(d->dtype, X_dev, ws, d->B, d->C_in, CSx, sm, st));
    XC_LAUNCH(K_ZERO_GAPS, st, launch_zero_gap_slices(ws, xslice, d->B, sm, st));
    float *T3 = reinterpret_cast<float *>(ws + xb + pb);
    void *dy_slices = ws + xb + pb + tb;
    if (vol_dy_in_place(v, g, E, dY_dev)) {
        P.dY = dY_dev;
    } else {
        if (d->layout == XCONV_NHWC)
            XC_LAUNCH(K_REPACK, st, launch_dy_slices_nhwc(d->dtype, dY_dev, dy_slices, d->B, d->C_out, g.Do, g.period, P.Ho * P.Wo, pitch, st));
        else
            XC_LAUNCH(K_REPACK, st, launch_dy_slices(d->dtype, dY_dev, dy_slices, d->B, d->C_out, g.Do, g.period, P.Ho * P.Wo, pitch, st));
        P.dY = dy_slices;
    }
    float *part0 = reinterpret_cast<float *>(ws + xb);
    for (int kz = 0; kz < v->kD; ++kz) {
        const void *A = ws + vol_offset_slices(g, kz) * xslice;
        P.A = A;
        P.part = part0 + (size_t)kz * P.S * (tile / sizeof(float));
        if (E.ws) {
            E.Wp.dY = P.dY;
            E.Wp.A = A;
            E.Wp.part = P.part;
            XC_LAUNCH(K_CORR, st, launch_ws_plan(d->dtype, E, st));
        } else {
            XC_LAUNCH(K_CORR, st, launch_corr(d->dtype, P, st));
        }
    }
    P.part = part0;
    if (reduce_expand_fused(P, false, true, d->C_in, d->r, 0)) {
        XC_LAUNCH(K_PASS2, st, launch_reduce_expand(P, nullptr, true, dW_dev, d->C_in, d->r, false, 0, 0, v->kD, st));
        return XCONV_OK;
    }
    XC_LAUNCH(K_REDUCE, st, launch_reduce(P, st, nullptr, 0, 0, 0, T3, v->kD));
    XC_LAUNCH(K_EXPAND, st, launch_expand(P, nullptr, dW_dev, d->C_in, d->r, st, false, T3, v->kD * P.K2));
    return XCONV_OK;
}

xconv_status xconv3d_xt_unpack(const xconv3d_desc *v, const void *Xt_dev, float *out_dev, void *stream)
{
    xconv_status s = xconv3d_check_desc(v);
    if (s != XCONV_OK) return s;
    if (!Xt_dev || !out_dev) return XCONV_EINVAL;
    const xconv_desc *d = &v->l;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const Vol g = vol_of(v);
    XC_LAUNCH(K_UNPACK, st, launch_unpack_slices(d->dtype, Xt_dev, out_dev, d->B, d->r, round_up(d->r, 16), vol_map(v, g), st));
    return XCONV_OK;
}

// ---- probing vectors over pixels and channels (the estimator as the paper states it) ---------------
// Composed from the kernels above.  Z [K = C_in*H*W, r] is drawn into images of K storage values
// (image j = probing vector j).
//   forward:  Xbar[b,j] = sum_k X[b,k] Z[k,j] is the exact-gradient path of a 1x1 layer with one
//             image, B output channels (the rows of X), r input channels (the probing vectors)
//             and K pixels;
//   backward: Lt[p,j] = sum_b dY[b,p] Xbar[b,j]/r is the channel probe of a single image with B
//             channels and P = C_out*H'*W' pixels, with Xbar/r as its probing matrix; brought into
//             planes L[j,m,oy,ox] it is the residual of a batch of r images whose activations are
//             the probing vectors, and dW is the exact-gradient path of that batch.
// Independent probing (every input channel with r probing vectors of its own, Sec. 3) runs the same
// steps with R = C_in*r vectors that are block diagonal over the channels: vector n*r + j is column j
// of Z on the rows of channel n and zero elsewhere, and the factor stays 1/r.
namespace {

struct PixelGeom {
    long long K, P;      // values per image of X and of dY
    int R;               // values of Xbar per image: r, or C_in*r with independent probing
    int G;               // independent probing: input channels per pass of the backward products (else 0)
    int Rb;              // probing vectors of one pass of the backward products: r, or G*r
    int CS;              // Rb rounded up to 16: images of L and of Z in one pass
    xconv_desc fwd;      // 1x1 layer of the forward product
    xconv_desc probe;    // single-image channel probe of the backward pass (B channels)
    xconv_desc bwd;      // batch of CS images of the shifted product
    size_t zimg_f, zimg_b, xs, lt, l, probe_ws, dwg, exact_ws;
    bool per_channel;    // independent probing, forward: one product per input channel from the r vectors of Z itself
    size_t zimg_c;       // ... and the bytes of those r vectors
};

xconv_status pixel_geom(const xconv_desc *d, bool indep, PixelGeom &g)
{
    xconv_status s = xconv_check_desc(d);
    if (s != XCONV_OK) return s;
    if (d->probe == XCONV_USER_Z) return XCONV_EUNSUPPORTED;
    if (indep && d->keep_q15 != 0) return XCONV_EUNSUPPORTED;
    if ((long long)d->C_in * d->r > (1LL << 24)) return XCONV_EUNSUPPORTED;
    const int Ho = out_extent(d->H, d->kH, d->stride_h, d->pad_h), Wo = out_extent(d->W, d->kW, d->stride_w, d->pad_w);
    g.K = (long long)d->C_in * d->H * d->W;
    g.P = (long long)d->C_out * Ho * Wo;
    if (g.K > (1LL << 28) || g.P > (1LL << 28)) return XCONV_EUNSUPPORTED;
    g.R = indep ? d->C_in * d->r : d->r;
    // independent probing, backward: groups of input channels, 16 (one block of channel slots of the shifted product)
    // or, for few vectors per channel, as many as give a pass about 256 vectors (a pass has fixed costs); at most 1024
    // probing vectors per pass
    g.G = 0;
    if (indep) {
        g.G = 256 / d->r > 16 ? 256 / d->r / 16 * 16 : 16;
        if (g.G > 1024 / d->r) g.G = 1024 / d->r;
        if (g.G > d->C_in) g.G = d->C_in;
    }
    g.Rb = indep ? g.G * d->r : d->r;
    g.CS = round_up(g.Rb, 16);
    const size_t eb = elem_bytes(d->dtype);
    g.fwd = *d;
    g.fwd.B = 1; g.fwd.C_out = d->B; g.fwd.C_in = g.R; g.fwd.H = d->C_in * d->H; g.fwd.W = d->W;
    g.fwd.kH = g.fwd.kW = 1; g.fwd.stride_h = g.fwd.stride_w = 1; g.fwd.pad_h = g.fwd.pad_w = 0;
    // the two products see rows of K (or P) contiguous values whatever their order; only the shifted product
    // looks at the layout (of L, which inherits dY's)
    g.fwd.layout = XCONV_NCHW;
    g.probe = *d;
    g.probe.B = 1; g.probe.C_in = d->B; g.probe.r = g.Rb; g.probe.probe = XCONV_USER_Z; g.probe.layout = XCONV_NCHW;
    g.bwd = *d;
    g.bwd.B = g.CS;
    if (indep) g.bwd.C_in = g.G;
    if (xconv_check_desc(&g.fwd) != XCONV_OK || xconv_check_desc(&g.probe) != XCONV_OK || xconv_check_desc(&g.bwd) != XCONV_OK)
        return XCONV_EUNSUPPORTED;
    g.zimg_f = align_up((size_t)g.R * g.K * eb, 256);
    g.zimg_b = align_up((size_t)g.CS * d->H * d->W * round_up(g.bwd.C_in, 16) * eb, 256);   // channels-last, padded channels
    g.xs = align_up((size_t)d->B * g.Rb * sizeof(float), 256);
    g.lt = align_up((size_t)g.P * g.CS * eb, 256);
    g.l = g.lt;
    g.probe_ws = z_bytes(&g.probe) + zfrag_bytes(&g.probe);
    g.dwg = indep ? align_up((size_t)d->C_out * g.G * d->kH * d->kW * sizeof(float), 256) : 0;
    g.exact_ws = xconv_workspace_bytes(&g.bwd, XCONV_OP_EXACT);
    if (indep && d->C_in % g.G != 0) {
        // the last pass has fewer channels: its shifted product may plan differently
        xconv_desc last = g.bwd;
        last.C_in = d->C_in % g.G;
        last.B = round_up(last.C_in * d->r, 16);
        const size_t w = xconv_workspace_bytes(&last, XCONV_OP_EXACT);
        if (w == 0) g.exact_ws = 0;
        else if (w > g.exact_ws) g.exact_ws = w;
    }
    // rows of one channel are contiguous in NCHW only, and the product wants them in whole 16-byte vectors
    g.per_channel = indep && d->layout == XCONV_NCHW && d->C_in <= kMaxGridZ && pixel_fwd_ok(d->dtype, (long long)d->H * d->W, nullptr);   // (one grid row per channel)
    g.zimg_c = align_up((size_t)d->r * g.K * eb, 256);
    return XCONV_OK;
}

size_t pixel_xbar_bytes(const xconv_desc *d, bool indep)
{
    PixelGeom g;
    if (pixel_geom(d, indep, g) != XCONV_OK) return 0;
    return (size_t)d->B * g.R * sizeof(float);
}

size_t pixel_workspace_bytes(const xconv_desc *d, bool indep, int op)
{
    PixelGeom g;
    if (pixel_geom(d, indep, g) != XCONV_OK) return 0;
    if (op == XCONV_OP_PROBE) {
        // the product kernel's partial sums, or (rows of X that are not whole 16-byte vectors) the scratch of the
        // exact-gradient path of the equivalent 1x1 layer
        // (an X that is not 16-byte aligned takes the block-diagonal route at run time: room for both)
        size_t alt = 0;
        if (g.per_channel)
            alt = g.zimg_c + align_up(pixel_fwd_indep_partial_bytes(d->dtype, (long long)d->H * d->W, d->C_in, d->B, d->r), 256);
        if (pixel_fwd_ok(d->dtype, g.K, nullptr)) {
            const size_t w = g.zimg_f + align_up(pixel_fwd_partial_bytes(d->dtype, g.K, d->B, g.R), 256);
            return w > alt ? w : alt;
        }
        const size_t w = xconv_workspace_bytes(&g.fwd, XCONV_OP_EXACT);
        if (w == 0) return 0;
        return g.zimg_f + w > alt ? g.zimg_f + w : alt;
    }
    if (op == XCONV_OP_ESTIMATE) {
        return g.exact_ws ? g.zimg_b + g.xs + g.lt + g.l + align_up(g.probe_ws, 256) + g.dwg + g.exact_ws : 0;
    }
    return 0;
}

xconv_status pixel_probe_fwd(const xconv_desc *d, bool indep, const void *X_dev, float *Xbar_dev, void *ws_dev, size_t ws_bytes,
                             void *stream)
{
    PixelGeom g;
    xconv_status s = pixel_geom(d, indep, g);
    if (s != XCONV_OK) return s;
    if (!X_dev || !Xbar_dev || !ws_dev) return XCONV_EINVAL;
    if (!aligned16(X_dev) || !aligned16(ws_dev) || (reinterpret_cast<uintptr_t>(Xbar_dev) & 3u) != 0) return XCONV_EINVAL;
    const size_t need = pixel_workspace_bytes(d, indep, XCONV_OP_PROBE);
    if (need == 0) return XCONV_EUNSUPPORTED;
    if (ws_bytes < need) return XCONV_EWORKSPACE;
    hipStream_t st = static_cast<hipStream_t>(stream);
    char *ws = static_cast<char *>(ws_dev);
    if (g.per_channel && pixel_fwd_ok(d->dtype, (long long)d->H * d->W, X_dev)) {
        // the r vectors of Z; channel n's product reads their rows of channel n
        XC_LAUNCH(K_GEN_ZIMG, st, launch_gen_zimg(d->dtype, ws, g.K, d->r, d->r, probe_code(d), d->seed, d->C_in, 0, 0, 0, d->C_in, st));
        XC_LAUNCH(K_PIXEL_FWD, st, launch_pixel_fwd_indep(d->dtype, X_dev, ws, reinterpret_cast<float *>(ws + g.zimg_c), Xbar_dev,
                                                          (long long)d->H * d->W, d->C_in, d->B, d->r, st));
        return XCONV_OK;
    }
    // probing vectors as rows in the order X keeps its values in: (n, y, x), or (y, x, n) for channels-last
    XC_LAUNCH(K_GEN_ZIMG, st, launch_gen_zimg(d->dtype, ws, g.K, d->r, g.R, probe_code(d), d->seed, d->C_in,
                                              d->layout == XCONV_NHWC ? d->C_in : 0, indep, 0, d->C_in, st));
    if (pixel_fwd_ok(d->dtype, g.K, X_dev)) {
        XC_LAUNCH(K_PIXEL_FWD, st, launch_pixel_fwd(d->dtype, X_dev, ws, reinterpret_cast<float *>(ws + g.zimg_f), Xbar_dev, g.K, d->B,
                                                    g.R, st));
        return XCONV_OK;
    }
    // rows of X in the role of dY (B channels of one image), the probing vectors in the role of the activation
    return xconv_dw_exact(&g.fwd, X_dev, ws, Xbar_dev, ws + g.zimg_f, ws_bytes - g.zimg_f, stream);
}

xconv_status pixel_dw_estimate(const xconv_desc *d, bool indep, const void *dY_dev, const float *Xbar_dev, float *dW_dev,
                               void *ws_dev, size_t ws_bytes, void *stream)
{
    PixelGeom g;
    xconv_status s = pixel_geom(d, indep, g);
    if (s != XCONV_OK) return s;
    if (!dY_dev || !Xbar_dev || !dW_dev || !ws_dev) return XCONV_EINVAL;
    if (!aligned16(dY_dev) || !aligned16(ws_dev) || (reinterpret_cast<uintptr_t>(dW_dev) & 3u) != 0 ||
        (reinterpret_cast<uintptr_t>(Xbar_dev) & 3u) != 0)
        return XCONV_EINVAL;
    const size_t need = pixel_workspace_bytes(d, indep, XCONV_OP_ESTIMATE);
    if (need == 0) return XCONV_EUNSUPPORTED;
    if (ws_bytes < need) return XCONV_EWORKSPACE;
    hipStream_t st = static_cast<hipStream_t>(stream);
    char *ws = static_cast<char *>(ws_dev);
    char *zimg = ws;
    float *xs = reinterpret_cast<float *>(ws + g.zimg_b);
    char *lt = ws + g.zimg_b + g.xs;
    char *l = lt + g.lt;
    char *pws = l + g.l;
    float *dwg = reinterpret_cast<float *>(pws + align_up(g.probe_ws, 256));
    char *xws = reinterpret_cast<char *>(dwg) + g.dwg;
    const size_t xws_bytes = ws_bytes - (size_t)(xws - ws);
    if (indep) {
        // one pass per group of input channels: its probing vectors are block diagonal over the group's channels, which
        // are the channel slots (a multiple of 16) of the images the shifted product reads
        const int K2 = d->kH * d->kW;
        for (int n0 = 0; n0 < d->C_in; n0 += g.G) {
            const int Gc = d->C_in - n0 < g.G ? d->C_in - n0 : g.G;
            const int Rg = Gc * d->r, CSg = round_up(Rg, 16);
            xconv_desc probe_g = g.probe, bwd_g = g.bwd;
            probe_g.r = Rg;
            bwd_g.B = CSg;
            bwd_g.C_in = Gc;
            XC_LAUNCH(K_GEN_ZIMG, st, launch_gen_zimg(d->dtype, zimg, g.K, d->r, CSg, probe_code(d), d->seed, d->C_in, round_up(Gc, 16), 1, n0, Gc, st));
            XC_LAUNCH(K_SCALE, st, launch_scale_cols(Xbar_dev, xs, d->B, g.R, n0 * d->r, Rg, 1.0f / (float)d->r, st));
            s = probe_impl(&probe_g, (int)g.P, (int)g.P, SliceMap{}, dY_dev, lt, xs, pws, g.probe_ws, st);
            if (s != XCONV_OK) return s;
            XC_LAUNCH(K_REPACK, st, launch_to_nchw(d->dtype, lt, l, 1, CSg, (int)g.P, (int)g.P, st));
            const bool whole = Gc == d->C_in;
            s = exact_impl(&bwd_g, l, nullptr, zimg, whole ? dW_dev : dwg, xws, xws_bytes, stream);
            if (s != XCONV_OK) return s;
            if (!whole) XC_LAUNCH(K_SCALE, st, launch_scatter_channels(dwg, dW_dev, d->C_out, d->C_in, K2, n0, Gc, st));
        }
        return XCONV_OK;
    }
    // Z[s] again (Alg. 1 backward step 2), CS images, channels-last as the correlation reads an activation:
    // the images past r are zero like the matching images of L
    XC_LAUNCH(K_GEN_ZIMG, st, launch_gen_zimg(d->dtype, zimg, g.K, d->r, g.CS, probe_code(d), d->seed, d->C_in, round_up(d->C_in, 16),
                                              0, 0, d->C_in, st));
    // Lt[p, j] = sum_b dY[b, p] Xbar[b, j] / r, rounded to the storage type (Alg. 1 backward step 3); p runs over
    // an image of dY in its own order, so the images of L come out in dY's layout.  The factor 1/r goes on Xbar where
    // the product brings it into fragment order, or in a launch of its own for the shapes that do not pass there
    const float inv_r = 1.0f / (float)d->r;
    const bool zfused = probe_scales_z(&g.probe, (int)g.P, dY_dev, pws);
    if (!zfused) XC_LAUNCH(K_SCALE, st, launch_scale(Xbar_dev, xs, d->B * g.R, inv_r, st));
    s = probe_impl(&g.probe, (int)g.P, (int)g.P, SliceMap{}, dY_dev, lt, zfused ? Xbar_dev : xs, pws, g.probe_ws, st, zfused ? inv_r : 1.0f);
    if (s != XCONV_OK) return s;
    XC_LAUNCH(K_REPACK, st, launch_to_nchw(d->dtype, lt, l, 1, g.CS, (int)g.P, (int)g.P, st));
    // dw_i = tr(L T_{-k(i)} Z) (Alg. 1 backward step 4; the factor 1/r is already in L)
    s = exact_impl(&g.bwd, l, nullptr, zimg, dW_dev, xws, xws_bytes, stream);
    if (s != XCONV_OK || d->keep_q15 == 0) return s;
    // block-sparse probes: 1/nnz(Z_n) per input channel in place of the 1/r that L carries (Eq. (8))
    XC_LAUNCH(K_SCALE, st, launch_nnz_rescale(dW_dev, d->C_out, d->C_in, d->kH * d->kW, d->r, probe_code(d), d->seed, st));
    return XCONV_OK;
}

}  // namespace

size_t xconv_pixel_xbar_bytes(const xconv_desc *d) { return pixel_xbar_bytes(d, false); }
size_t xconv_pixel_workspace_bytes(const xconv_desc *d, int op) { return pixel_workspace_bytes(d, false, op); }
xconv_status xconv_pixel_probe_fwd(const xconv_desc *d, const void *X_dev, float *Xbar_dev, void *ws_dev, size_t ws_bytes,
                                   void *stream)
{
    return pixel_probe_fwd(d, false, X_dev, Xbar_dev, ws_dev, ws_bytes, stream);
}
xconv_status xconv_pixel_dw_estimate(const xconv_desc *d, const void *dY_dev, const float *Xbar_dev, float *dW_dev, void *ws_dev,
                                     size_t ws_bytes, void *stream)
{
    return pixel_dw_estimate(d, false, dY_dev, Xbar_dev, dW_dev, ws_dev, ws_bytes, stream);
}

size_t xconv_pixel_indep_xbar_bytes(const xconv_desc *d) { return pixel_xbar_bytes(d, true); }
size_t xconv_pixel_indep_workspace_bytes(const xconv_desc *d, int op) { return pixel_workspace_bytes(d, true, op); }
xconv_status xconv_pixel_indep_probe_fwd(const xconv_desc *d, const void *X_dev, float *Xbar_dev, void *ws_dev, size_t ws_bytes,
                                         void *stream)
{
    return pixel_probe_fwd(d, true, X_dev, Xbar_dev, ws_dev, ws_bytes, stream);
}
xconv_status xconv_pixel_indep_dw_estimate(const xconv_desc *d, const void *dY_dev, const float *Xbar_dev, float *dW_dev, void *ws_dev,
                                           size_t ws_bytes, void *stream)
{
    return pixel_dw_estimate(d, true, dY_dev, Xbar_dev, dW_dev, ws_dev, ws_bytes, stream);
}

// ---- ReLU that keeps signs only -----------------------------------------------------
size_t xconv_relu_mask_bytes(long long n) { return n <= 0 ? 0 : (size_t)((n + 63) / 64) * 8; }

xconv_status xconv_relu_fwd(int dtype, const void *X_dev, void *Y_dev, void *mask_dev, long long n, void *stream)
{
    if (dtype < XCONV_F32 || dtype > XCONV_F16 || n < 0) return XCONV_EINVAL;
    if (n == 0) return XCONV_OK;
    if (!X_dev || !Y_dev || !mask_dev) return XCONV_EINVAL;
    if (!aligned16(X_dev) || !aligned16(Y_dev) || (reinterpret_cast<uintptr_t>(mask_dev) & 7u) != 0) return XCONV_EINVAL;
    if (n > (1LL << 40)) return XCONV_EUNSUPPORTED;
    hipStream_t st = static_cast<hipStream_t>(stream);
    XC_LAUNCH(K_RELU, st, launch_relu_sign_fwd(dtype, X_dev, Y_dev, mask_dev, n, st));
    return XCONV_OK;
}

xconv_status xconv_relu_bwd(int dtype, const void *dY_dev, const void *mask_dev, void *dX_dev, long long n, void *stream)
{
    if (dtype < XCONV_F32 || dtype > XCONV_F16 || n < 0) return XCONV_EINVAL;
    if (n == 0) return XCONV_OK;
    if (!dY_dev || !dX_dev || !mask_dev) return XCONV_EINVAL;
    if (!aligned16(dY_dev) || !aligned16(dX_dev) || (reinterpret_cast<uintptr_t>(mask_dev) & 7u) != 0) return XCONV_EINVAL;
    if (n > (1LL << 40)) return XCONV_EUNSUPPORTED;
    hipStream_t st = static_cast<hipStream_t>(stream);
    XC_LAUNCH(K_RELU, st, launch_relu_sign_bwd(dtype, dY_dev, mask_dev, dX_dev, n, st));
    return XCONV_OK;
}

xconv_status xconv_diag_mfma_rate(int dtype, int iters, float *out_dev, size_t out_bytes, double *flops, void *stream)
{
    if (dtype < XCONV_F32 || dtype > XCONV_F16 || iters < 1 || iters > (1 << 24) || !out_dev) return XCONV_EINVAL;
    if (out_bytes < XCONV_DIAG_OUT_BYTES) return XCONV_EWORKSPACE;
    if (reinterpret_cast<uintptr_t>(out_dev) & 3u) return XCONV_EINVAL;
    if (flops) *flops = mfma_rate_flops(dtype, iters);
    hipStream_t st = static_cast<hipStream_t>(stream);
    XC_LAUNCH(K_DIAG, st, launch_mfma_rate(dtype, out_dev, iters, st));
    return XCONV_OK;
}

void xconv_prof_enable(int on)
{
    std::lock_guard<std::mutex> lk(g_prof_mu);
    g_prof_on = on != 0;
}

int xconv_prof_collect(int32_t *kernel_ids, float *ms, int max)
{
    std::lock_guard<std::mutex> lk(g_prof_mu);
    int n = 0;
    for (ProfRec &r : g_prof) {
        float t = 0.f;
        if (hipEventSynchronize(r.b) == hipSuccess && hipEventElapsedTime(&t, r.a, r.b) == hipSuccess && n < max) {
            if (kernel_ids) kernel_ids[n] = r.id;
            if (ms) ms[n] = t;
            ++n;
        }
        (void)hipEventDestroy(r.a);
        (void)hipEventDestroy(r.b);
    }
    g_prof.clear();
    return n;
}

const char *xconv_prof_kernel_name(int id)
{
    switch (id) {
    case K_GEN_Z: return "gen_z_kernel";
    case K_PROBE: return "probe_kernel";
    case K_PROBE_GENERIC: return "probe_generic_kernel";
    case K_CORR: return "corr_kernel";
    case K_REDUCE: return "reduce_partials_kernel";
    case K_EXPAND: return "expand_kernel";
    case K_PASS2: return "pass2_kernel";
    case K_DIAG: return "mfma_rate_kernel";
    case K_TO_NHWC: return "to_nhwc_kernel";
    case K_UNPACK: return "unpack_kernel";
    case K_REPACK: return "repack_planes_kernel";
    case K_PACK_Z: return "pack_z_kernel";
    case K_CONV: return "conv_gemm_kernel";
    case K_ZERO_GAPS: return "zero_gap_slices_kernel";
    case K_GEN_ZIMG: return "gen_zimg_kernel";
    case K_SCALE: return "scale_kernel";
    case K_PIXEL_FWD: return "pixel_fwd_kernel";
    case K_RELU: return "relu_sign_kernel";
    default: return "unknown";
    }
}

const char *xconv_status_string(int status)
{
    switch (status) {
    case XCONV_OK: return "ok";
    case XCONV_EINVAL: return "invalid argument";
    case XCONV_EUNSUPPORTED: return "unsupported configuration";
    case XCONV_EWORKSPACE: return "workspace too small";
    case XCONV_EHIP: return "HIP runtime error";
    default: return "unknown status";
    }
}

}  // extern "C"
