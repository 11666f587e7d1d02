// C ABI of the convolution passes: descriptor validation and kernel choice.
#include <cstdio>
#include <cstring>
#include <mutex>

#include "mi3d_internal.h"

namespace mi3d {

static thread_local int g_last_hip_error = 0;

void note_hip_error(hipError_t e) { g_last_hip_error = (int)e; }

int check_launch() {
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) {
        note_hip_error(e);
        return MI3D_ERR_HIP;
    }
    return MI3D_OK;
}

int make_geom(const mi3d_conv_desc* d, Geom* g) {
    if (!d) return MI3D_ERR_INVALID_ARG;
    if (d->N <= 0 || d->D <= 0 || d->H <= 0 || d->W <= 0 || d->Cin <= 0 || d->Cout <= 0) return MI3D_ERR_INVALID_ARG;
    if (d->kD <= 0 || d->kH <= 0 || d->kW <= 0 || d->sD <= 0 || d->sH <= 0 || d->sW <= 0) return MI3D_ERR_INVALID_ARG;
    if (d->pD < 0 || d->pH < 0 || d->pW < 0) return MI3D_ERR_INVALID_ARG;
    if (d->D + 2 * d->pD < d->kD || d->H + 2 * d->pH < d->kH || d->W + 2 * d->pW < d->kW) return MI3D_ERR_INVALID_ARG;
    if (d->dtype != MI3D_F32 && d->dtype != MI3D_BF16) return MI3D_ERR_UNSUPPORTED;
    g->N = d->N; g->D = d->D; g->H = d->H; g->W = d->W; g->Cin = d->Cin;
    g->Cout = d->Cout; g->kD = d->kD; g->kH = d->kH; g->kW = d->kW;
    g->sD = d->sD; g->sH = d->sH; g->sW = d->sW; g->pD = d->pD; g->pH = d->pH; g->pW = d->pW;
    g->Do = (d->D + 2 * d->pD - d->kD) / d->sD + 1;
    g->Ho = (d->H + 2 * d->pH - d->kH) / d->sH + 1;
    g->Wo = (d->W + 2 * d->pW - d->kW) / d->sW + 1;
    g->dtype = d->dtype;
    // element counts must stay addressable with 63-bit indices and sane grids
    const long long lim = 1ll << 40;
    if (g->in_voxels() * g->Cin > lim || g->out_voxels() * g->Cout > lim || g->w_elems() > (1ll << 31)) return MI3D_ERR_UNSUPPORTED;
    return MI3D_OK;
}

static bool aligned16(const void* p) { return ((uintptr_t)p & 15) == 0; }

enum Kernel {
    K_DIRECT = 0, K_SP, K_WGRAD_MFMA, K_S2_FWD, K_WGRAD_S2, K_DGRAD_S2, K_C4_FWD, K_C4_DGRAD, K_C4_WGRAD, K_POINTWISE,
    K_EMBED_C, K_EMBED_S, K_EMBED_K2, K_K2, K_F32
};

static Kernel choose(const Geom& g, int pass) {
    if (f32_supported(g, pass)) return K_F32;
    if (pointwise_supported(g)) return K_POINTWISE;
    if (pass == MI3D_PASS_WGRAD && wgrad_mfma_supported(g)) return K_WGRAD_MFMA;
    if (pass == MI3D_PASS_WGRAD && wgrad_s2_supported(g)) return K_WGRAD_S2;
    if (sp_supported(g, pass)) return K_SP;
    if (pass == MI3D_PASS_FWD && s2_fwd_supported(g)) return K_S2_FWD;
    if (pass == MI3D_PASS_DGRAD && dgrad_s2_supported(g)) return K_DGRAD_S2;
    if (pass == MI3D_PASS_FWD && c4_fwd_supported(g)) return K_C4_FWD;
    if (pass == MI3D_PASS_DGRAD && c4_dgrad_supported(g)) return K_C4_DGRAD;
    if (pass == MI3D_PASS_WGRAD && c4_wgrad_supported(g)) return K_C4_WGRAD;
    if (k2_supported(g, pass)) return K_K2;
    if (embed_c_supported(g, pass)) return K_EMBED_C;
    if (embed_s_supported(g, pass)) return K_EMBED_S;
    if (embed_k2_supported(g, pass)) return K_EMBED_K2;
    return K_DIRECT;
}

static const char* kernel_name(Kernel k) {
    switch (k) {
        case K_DIRECT: return "direct";
        case K_SP: return "mfma_plane_stream";
        case K_WGRAD_MFMA: return "mfma_wgrad_plane_stream";
        case K_S2_FWD: return "mfma_stride2_plane_stream";
        case K_WGRAD_S2: return "mfma_wgrad_stride2";
        case K_DGRAD_S2: return "mfma_dgrad_stride2_parity";
        case K_POINTWISE: return "valu_pointwise_head";
        case K_C4_FWD: return "mfma_cin4_folded_taps";
        case K_C4_DGRAD: return "mfma_dgrad_cin4_folded_taps";
        case K_C4_WGRAD: return "mfma_wgrad_cin4_folded_taps";
        case K_EMBED_C: return "mfma_via_channel_padding";
        case K_EMBED_S: return "mfma_via_unit_stride";
        case K_EMBED_K2: return "mfma_via_k3s2_embedding";
        case K_K2: return "mfma_k2s2_panel_gemm";
        case K_F32: return "mfma_f32_gather";
        default: return "none";
    }
}

static size_t kernel_workspace(Kernel k, const Geom& g, int pass) {
    switch (k) {
        case K_DIRECT: return direct_workspace_bytes(g, pass);
        case K_SP: return sp_workspace_bytes(g, pass);
        case K_WGRAD_MFMA: return wgrad_mfma_workspace_bytes(g);
        case K_S2_FWD: return s2_fwd_workspace_bytes(g);
        case K_WGRAD_S2: return wgrad_s2_workspace_bytes(g);
        case K_DGRAD_S2: return dgrad_s2_workspace_bytes(g);
        case K_C4_FWD: return c4_fwd_workspace_bytes(g);
        case K_C4_DGRAD: return c4_dgrad_workspace_bytes(g);
        case K_C4_WGRAD: return c4_wgrad_workspace_bytes(g);
        case K_POINTWISE: return pointwise_workspace_bytes(g, pass);
        case K_EMBED_C: return embed_c_workspace_bytes(g, pass);
        case K_EMBED_S: return embed_s_workspace_bytes(g, pass);
        case K_EMBED_K2: return embed_k2_workspace_bytes(g, pass);
        case K_K2: return k2_workspace_bytes(g, pass);
        case K_F32: return f32_workspace_bytes(g, pass);
    }
    return 0;
}

// a, b, out per pass: fwd (x, w, y), dgrad (dy, w, dx), wgrad (x, dy, dw)
static int run_kernel(Kernel k, const Geom& g, int pass, const void* a, const void* b, void* out, void* ws, size_t ws_bytes, hipStream_t s) {
    switch (k) {
        case K_DIRECT:
            if (pass == MI3D_PASS_FWD) return direct_fwd(g, a, b, out, s);
            if (pass == MI3D_PASS_DGRAD) return direct_dgrad(g, a, b, out, s);
            return direct_wgrad(g, a, b, (float*)out, ws, ws_bytes, s);
        case K_SP: return sp_conv(g, pass, a, b, out, ws, ws_bytes, s);
        case K_WGRAD_MFMA: return wgrad_mfma(g, a, b, (float*)out, ws, ws_bytes, s);
        case K_S2_FWD: return s2_fwd(g, a, b, out, ws, ws_bytes, s);
        case K_WGRAD_S2: return wgrad_s2(g, a, b, (float*)out, ws, ws_bytes, s);
        case K_DGRAD_S2: return dgrad_s2(g, a, b, out, ws, ws_bytes, s);
        case K_C4_FWD: return c4_fwd(g, a, b, out, ws, ws_bytes, s);
        case K_C4_DGRAD: return c4_dgrad(g, a, b, out, ws, ws_bytes, s);
        case K_C4_WGRAD: return c4_wgrad(g, a, b, (float*)out, ws, ws_bytes, s);
        case K_POINTWISE: return pointwise_conv(g, pass, a, b, out, ws, ws_bytes, s);
        case K_EMBED_C: return embed_c_conv(g, pass, a, b, out, ws, ws_bytes, s);
        case K_EMBED_S: return embed_s_conv(g, pass, a, b, out, ws, ws_bytes, s);
        case K_EMBED_K2: return embed_k2_conv(g, pass, a, b, out, ws, ws_bytes, s);
        case K_K2: return k2_conv(g, pass, a, b, out, ws, ws_bytes, s);
        case K_F32:
            if (pass == MI3D_PASS_WGRAD) return f32_wgrad(g, a, b, (float*)out, ws, ws_bytes, s);
            return f32_conv(g, pass, a, b, out, ws, ws_bytes, s);
    }
    return MI3D_ERR_UNSUPPORTED;
}

// Kernels that apply the optional epilogue of the geometry themselves (the others are followed by one elementwise pass)
static bool fuses_epilogue(Kernel k, const Geom& g, int pass) {
    if (k == K_F32) return pass != MI3D_PASS_WGRAD;
    if (pass == MI3D_PASS_FWD) return k == K_SP || k == K_S2_FWD || k == K_C4_FWD;
    if (pass == MI3D_PASS_DGRAD) return (k == K_SP && sp_fuses_dgrad_factor(g)) || (k == K_DGRAD_S2 && dgrad_s2_fuses_factor(g)) || k == K_POINTWISE;
    return false;
}

// the kernels that take the tensor of x's shape as two halves along the channels
static bool pair_supported(const Geom& g, int pass) {
    if (g.Cin % 64) return false;
    const Kernel k = choose(g, pass);
    if (k == K_F32) return f32_takes_halves(g, pass);
    return pass == MI3D_PASS_WGRAD ? k == K_WGRAD_MFMA : k == K_SP;
}

// automatic choice for a geometry, used by the entry points and by fallbacks that re-enter with a derived geometry
size_t auto_workspace_bytes(const Geom& g, int pass) { return kernel_workspace(choose(g, pass), g, pass); }
int auto_conv(const Geom& g, int pass, const void* a, const void* b, void* out, void* ws, size_t ws_bytes, hipStream_t s) {
    return run_kernel(choose(g, pass), g, pass, a, b, out, ws, ws_bytes, s);
}

}  // namespace mi3d

using namespace mi3d;

extern "C" {

const char* mi3d_status_string(int status) {
    switch (status) {
        case MI3D_OK: return "ok";
        case MI3D_ERR_INVALID_ARG: return "invalid argument";
        case MI3D_ERR_UNSUPPORTED: return "unsupported dtype or shape";
        case MI3D_ERR_WORKSPACE: return "workspace too small";
        case MI3D_ERR_HIP: return "HIP runtime error";
        case MI3D_ERR_HOST_POOL: return "pinned host pool exhausted";
        case MI3D_ERR_OVER_BUDGET: return "device budget or arena exceeded";
        case MI3D_ERR_BAD_STATE: return "call not valid in this state";
        default: return "unknown status";
    }
}

int mi3d_last_hip_error(void) { return g_last_hip_error; }

int mi3d_conv3d_out_dims(const mi3d_conv_desc* desc, int* Do, int* Ho, int* Wo) {
    Geom g;
    int st = make_geom(desc, &g);
    if (st) return st;
    if (!Do || !Ho || !Wo) return MI3D_ERR_INVALID_ARG;
    *Do = g.Do; *Ho = g.Ho; *Wo = g.Wo;
    return MI3D_OK;
}

int mi3d_conv3d_kernel_name(const mi3d_conv_desc* desc, int pass, char* buf, size_t buf_len) {
    Geom g;
    int st = make_geom(desc, &g);
    if (st) return st;
    if (!buf || buf_len == 0 || pass < 0 || pass > 2) return MI3D_ERR_INVALID_ARG;
    Kernel k = choose(g, pass);
    // (the fp32 dispatcher hands 1x1x1 layers with a handful of output channels to VALU kernels of its own, and the
    // weight gradient of a layer with at most 4 input channels to a kernel that folds the taps into the block's columns)
    const char* name = kernel_name(k);
    if (k == K_F32 && pointwise_f32_supported(g)) name = "valu_pointwise_head_f32";
    else if (k == K_F32 && pass == MI3D_PASS_WGRAD && f32_wgrad_folds_taps(g)) name = "mfma_f32_wgrad_cin4_folded_taps";
    snprintf(buf, buf_len, "%s", name);
    return MI3D_OK;
}

size_t mi3d_conv3d_workspace_bytes(const mi3d_conv_desc* desc, int pass) {
    Geom g;
    if (make_geom(desc, &g) || pass < 0 || pass > 2) return 0;
    return auto_workspace_bytes(g, pass);
}

// slope / ref: optional LeakyReLU epilogue (forward: on y; data gradient: derivative factor from ref), 1 / null = none
static int conv_entry(const mi3d_conv_desc* desc, int pass, const void* a, const void* b, void* out, void* ws, size_t ws_bytes, void* stream,
                      float slope = 1.f, const void* ref = nullptr, const mi3d_view* xv = nullptr, const void* hi = nullptr, bool pair = false) {
    Geom g;
    int st = make_geom(desc, &g);
    if (st) return st;
    if (pair) {   // the tensor of x's shape comes as two halves along the channels
        if (!hi || !aligned16(hi)) return MI3D_ERR_INVALID_ARG;
        if (!pair_supported(g, pass)) return MI3D_ERR_UNSUPPORTED;
        g.hi = hi;
    }
    if (xv && xv->pitch) {   // the tensor of x's shape is a channel range of a wider tensor
        if (xv->pitch < 0 || xv->offset < 0 || xv->offset + g.Cin > xv->pitch || xv->pitch % 8 || xv->offset % 8) return MI3D_ERR_INVALID_ARG;
        if (choose(g, pass) != K_K2) return MI3D_ERR_UNSUPPORTED;
        g.x_pitch = xv->pitch;
        g.x_off = xv->offset;
    }
    if (!a || !b || !out || !aligned16(a) || !aligned16(b) || !aligned16(out) || !aligned16(ws)) return MI3D_ERR_INVALID_ARG;
    if (ws_bytes && !ws) return MI3D_ERR_INVALID_ARG;
    if (ws_bytes < mi3d_conv3d_workspace_bytes(desc, pass)) return MI3D_ERR_WORKSPACE;
    Kernel k = choose(g, pass);
    const bool epilogue = slope != 1.f;
    if (!epilogue) return run_kernel(k, g, pass, a, b, out, ws, ws_bytes, (hipStream_t)stream);
    if (!(slope >= 0.f && slope < 1.f) || (g.dtype != MI3D_BF16 && k != K_F32) || pass == MI3D_PASS_WGRAD) return MI3D_ERR_INVALID_ARG;
    if (pass == MI3D_PASS_DGRAD && (!ref || !aligned16(ref))) return MI3D_ERR_INVALID_ARG;
    Geom ge = g;
    ge.slope = slope;
    ge.ref = ref;
    if (fuses_epilogue(k, ge, pass)) return run_kernel(k, ge, pass, a, b, out, ws, ws_bytes, (hipStream_t)stream);
    st = run_kernel(k, g, pass, a, b, out, ws, ws_bytes, (hipStream_t)stream);
    if (st) return st;
    const long long n = pass == MI3D_PASS_FWD ? g.out_voxels() * g.Cout : g.in_voxels() * g.Cin;
    if (n % 8) return MI3D_ERR_UNSUPPORTED;
    if (pass == MI3D_PASS_FWD) return mi3d_leaky_relu_fwd(out, n, slope, stream);
    return mi3d_leaky_relu_bwd(out, ref, n, slope, stream);
}

int mi3d_conv3d_fwd(const mi3d_conv_desc* desc, const void* x, const void* w, void* y, void* ws, size_t ws_bytes, void* stream) {
    return conv_entry(desc, MI3D_PASS_FWD, x, w, y, ws, ws_bytes, stream);
}

int mi3d_conv3d_dgrad(const mi3d_conv_desc* desc, const void* dy, const void* w, void* dx, void* ws, size_t ws_bytes, void* stream) {
    return conv_entry(desc, MI3D_PASS_DGRAD, dy, w, dx, ws, ws_bytes, stream);
}

int mi3d_conv3d_wgrad(const mi3d_conv_desc* desc, const void* x, const void* dy, float* dw, void* ws, size_t ws_bytes, void* stream) {
    return conv_entry(desc, MI3D_PASS_WGRAD, x, dy, dw, ws, ws_bytes, stream);
}

// ---- weight gradient for callers that cannot allocate -------------------------------------------------------------
// The per-workgroup partial sums of the weight-gradient kernels (and their packed operands) go to a file-scope device
// array instead of a caller-provided workspace.  The array's name is only a host-side handle: its device address is
// looked up once per device with hipGetSymbolAddress and that pointer is what the kernels get.
static __device__ __align__(256) unsigned char scratch[MI3D_STATIC_SCRATCH_BYTES];
static std::mutex g_scratch_mutex;
static void* g_scratch_ptr[64] = {};   // per device; each device holds its own copy of the array at its own address

static int scratch_of_current_device(void** out) {
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) { note_hip_error(e); return MI3D_ERR_HIP; }
    if (dev < 0 || dev >= 64) return MI3D_ERR_UNSUPPORTED;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void* p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !p) { note_hip_error(e); return MI3D_ERR_HIP; }
        g_scratch_ptr[dev] = p;
    }
    *out = g_scratch_ptr[dev];
    return MI3D_OK;
}

size_t mi3d_static_scratch_bytes(void) { return MI3D_STATIC_SCRATCH_BYTES; }

int mi3d_conv3d_wgrad_static(const mi3d_conv_desc* desc, const void* x, const void* dy, float* dw, void* stream) {
    Geom g;
    int st = make_geom(desc, &g);
    if (st) return st;
    // sizes beyond the array are refused before anything is looked up or launched
    if (mi3d_conv3d_workspace_bytes(desc, MI3D_PASS_WGRAD) > (size_t)MI3D_STATIC_SCRATCH_BYTES) return MI3D_ERR_WORKSPACE;
    void* ws = nullptr;
    st = scratch_of_current_device(&ws);
    if (st) return st;
    // every kernel of the pass writes the part of the scratch it later reads, so nothing has to be cleared between calls
    return conv_entry(desc, MI3D_PASS_WGRAD, x, dy, dw, ws, (size_t)MI3D_STATIC_SCRATCH_BYTES, stream);
}

int mi3d_conv3d_fwd_view(const mi3d_conv_desc* desc, const void* x, const mi3d_view* xv, const void* w, void* y, void* ws, size_t ws_bytes, void* stream) {
    return conv_entry(desc, MI3D_PASS_FWD, x, w, y, ws, ws_bytes, stream, 1.f, nullptr, xv);
}

int mi3d_conv3d_dgrad_view(const mi3d_conv_desc* desc, const void* dy, const void* w, void* dx, const mi3d_view* dxv, void* ws, size_t ws_bytes, void* stream) {
    return conv_entry(desc, MI3D_PASS_DGRAD, dy, w, dx, ws, ws_bytes, stream, 1.f, nullptr, dxv);
}

int mi3d_conv3d_wgrad_view(const mi3d_conv_desc* desc, const void* x, const mi3d_view* xv, const void* dy, float* dw, void* ws, size_t ws_bytes, void* stream) {
    return conv_entry(desc, MI3D_PASS_WGRAD, x, dy, dw, ws, ws_bytes, stream, 1.f, nullptr, xv);
}

int mi3d_conv3d_dgrad_skip(const mi3d_conv_desc* desc, const void* dy, const void* w, const void* add, const void* a_in, float slope, void* dx,
                           void* ws, size_t ws_bytes, void* stream) {
    Geom g;
    int st = make_geom(desc, &g);
    if (st) return st;
    if (!dy || !w || !add || !a_in || !dx || !aligned16(dy) || !aligned16(w) || !aligned16(add) || !aligned16(a_in) || !aligned16(dx) || !aligned16(ws))
        return MI3D_ERR_INVALID_ARG;
    const Kernel k = choose(g, MI3D_PASS_DGRAD);
    if ((g.dtype != MI3D_BF16 && k != K_F32) || !(slope >= 0.f && slope <= 1.f) || (ws_bytes && !ws)) return MI3D_ERR_INVALID_ARG;
    if (ws_bytes < mi3d_conv3d_workspace_bytes(desc, MI3D_PASS_DGRAD)) return MI3D_ERR_WORKSPACE;
    if (k == K_F32 || (k == K_DGRAD_S2 && dgrad_s2_fuses_skip(g))) {
        Geom ge = g;
        ge.add = add; ge.ref = a_in; ge.slope = slope;
        return run_kernel(k, ge, MI3D_PASS_DGRAD, dy, w, dx, ws, ws_bytes, (hipStream_t)stream);
    }
    st = run_kernel(k, g, MI3D_PASS_DGRAD, dy, w, dx, ws, ws_bytes, (hipStream_t)stream);
    if (st) return st;
    if (g.Cin % 8) return MI3D_ERR_UNSUPPORTED;
    return mi3d_skip_grad(dx, add, g.Cin, 0, a_in, g.Cin, (size_t)g.in_voxels(), slope, stream);
}

int mi3d_conv3d_fwd_stats_supported(const mi3d_conv_desc* desc) {
    Geom g;
    if (make_geom(desc, &g)) return 0;
    const Kernel k = choose(g, MI3D_PASS_FWD);
    return (k == K_SP && sp_fuses_stats(g)) || (k == K_C4_FWD && c4_fwd_fuses_stats(g)) ? 1 : 0;
}

int mi3d_conv3d_fwd_stats(const mi3d_conv_desc* desc, const void* x, const void* x_hi, const void* w, void* y, float eps, float* stats,
                          void* ws, size_t ws_bytes, void* stream) {
    Geom g;
    int st = make_geom(desc, &g);
    if (st) return st;
    if (!x || !w || !y || !stats || !aligned16(x) || !aligned16(x_hi) || !aligned16(w) || !aligned16(y) || !aligned16(ws) || !(eps > 0.f))
        return MI3D_ERR_INVALID_ARG;
    if (ws_bytes && !ws) return MI3D_ERR_INVALID_ARG;
    if (!mi3d_conv3d_fwd_stats_supported(desc) || (x_hi && !pair_supported(g, MI3D_PASS_FWD))) return MI3D_ERR_UNSUPPORTED;
    if (ws_bytes < mi3d_conv3d_workspace_bytes(desc, MI3D_PASS_FWD)) return MI3D_ERR_WORKSPACE;
    g.hi = x_hi;
    g.stats = stats;
    g.stats_eps = eps;
    return run_kernel(choose(g, MI3D_PASS_FWD), g, MI3D_PASS_FWD, x, w, y, ws, ws_bytes, (hipStream_t)stream);
}

int mi3d_conv3d_dgrad_insums_supported(const mi3d_conv_desc* desc, int with_add) {
    Geom g;
    if (make_geom(desc, &g)) return 0;
    const Kernel k = choose(g, MI3D_PASS_DGRAD);
    if (with_add) return k == K_DGRAD_S2 && dgrad_s2_fuses_skip_sums(g) ? 1 : 0;
    return (k == K_SP && sp_fuses_bwd_sums(g)) || k == K_POINTWISE ? 1 : 0;
}

int mi3d_conv3d_dgrad_insums(const mi3d_conv_desc* desc, const void* dy, const void* w, const void* add, const void* a_in, float slope, void* dx,
                             float* sums, void* ws, size_t ws_bytes, void* stream) {
    Geom g;
    int st = make_geom(desc, &g);
    if (st) return st;
    if (!dy || !w || !a_in || !dx || !sums || !aligned16(dy) || !aligned16(w) || !aligned16(add) || !aligned16(a_in) || !aligned16(dx) ||
        !aligned16(ws) || !(slope > 0.f && slope <= 1.f))
        return MI3D_ERR_INVALID_ARG;
    if (ws_bytes && !ws) return MI3D_ERR_INVALID_ARG;
    if (!mi3d_conv3d_dgrad_insums_supported(desc, add ? 1 : 0)) return MI3D_ERR_UNSUPPORTED;
    if (ws_bytes < mi3d_conv3d_workspace_bytes(desc, MI3D_PASS_DGRAD)) return MI3D_ERR_WORKSPACE;
    g.add = add;
    g.ref = a_in;
    g.slope = slope;
    g.stats = sums;
    return run_kernel(choose(g, MI3D_PASS_DGRAD), g, MI3D_PASS_DGRAD, dy, w, dx, ws, ws_bytes, (hipStream_t)stream);
}

int mi3d_conv3d_pair_supported(const mi3d_conv_desc* desc, int pass) {
    Geom g;
    if (make_geom(desc, &g) || pass < 0 || pass > 2) return 0;
    return pair_supported(g, pass) ? 1 : 0;
}

int mi3d_conv3d_fwd_pair(const mi3d_conv_desc* desc, const void* x_lo, const void* x_hi, const void* w, void* y, float slope,
                         void* ws, size_t ws_bytes, void* stream) {
    return conv_entry(desc, MI3D_PASS_FWD, x_lo, w, y, ws, ws_bytes, stream, slope, nullptr, nullptr, x_hi, true);
}

int mi3d_conv3d_dgrad_pair(const mi3d_conv_desc* desc, const void* dy, const void* w, void* dx_lo, void* dx_hi,
                           void* ws, size_t ws_bytes, void* stream) {
    return conv_entry(desc, MI3D_PASS_DGRAD, dy, w, dx_lo, ws, ws_bytes, stream, 1.f, nullptr, nullptr, dx_hi, true);
}

int mi3d_conv3d_wgrad_pair(const mi3d_conv_desc* desc, const void* x_lo, const void* x_hi, const void* dy, float* dw,
                           void* ws, size_t ws_bytes, void* stream) {
    return conv_entry(desc, MI3D_PASS_WGRAD, x_lo, dy, dw, ws, ws_bytes, stream, 1.f, nullptr, nullptr, x_hi, true);
}

int mi3d_conv3d_fwd_lrelu(const mi3d_conv_desc* desc, const void* x, const void* w, void* y, float slope, void* ws, size_t ws_bytes, void* stream) {
    if (slope == 1.f) return MI3D_ERR_INVALID_ARG;
    return conv_entry(desc, MI3D_PASS_FWD, x, w, y, ws, ws_bytes, stream, slope, nullptr);
}

int mi3d_conv3d_dgrad_lrelu(const mi3d_conv_desc* desc, const void* dy, const void* w, const void* a_in, float slope, void* dx,
                            void* ws, size_t ws_bytes, void* stream) {
    if (slope == 1.f) return MI3D_ERR_INVALID_ARG;
    return conv_entry(desc, MI3D_PASS_DGRAD, dy, w, dx, ws, ws_bytes, stream, slope, a_in);
}

}  // extern "C"
