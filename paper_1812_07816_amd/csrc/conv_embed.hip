// Fallbacks that run a layer no tuned kernel covers through the stride-1
// 32-channel MFMA kernels by embedding its operands:
//   - few input channels (the network's first layer, Cin = 4): x and w are
//     zero-padded to 32 channels; results are sliced back;
//   - strided layers: the forward pass is the stride-1 result subsampled;
//     for the gradients dy is spread onto the stride-1 output grid (zeros in
//     between), after which dx and dw are exactly the stride-1 gradients.
// They trade extra MFMA work and one extra pass over a tensor for not falling
// back to the plain kernels; dedicated kernels replace them where it matters.
#include "mi3d_internal.h"

namespace mi3d {
namespace {

// dst[v][0..CP) = src[v][0..C) followed by zeros; one thread per 8 output channels
__global__ void __launch_bounds__(256) pad_channels_kernel(const uint16_t* __restrict__ src, uint16_t* __restrict__ dst,
                                                           long long voxels, int C, int CP) {
    const int per = CP / 8;
    long long idx = (long long)blockIdx.x * 256 + threadIdx.x;
    if (idx >= voxels * per) return;
    long long v = idx / per;
    int c0 = (int)(idx % per) * 8;
    uint16_t o[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) o[j] = (c0 + j < C) ? src[v * C + c0 + j] : (uint16_t)0;
    *(uint4*)(dst + v * CP + c0) = *(const uint4*)o;
}

// dst[v][0..C) = src[v][0..C) of CP-channel rows (T = uint16_t or float)
template <typename T>
__global__ void __launch_bounds__(256) slice_channels_kernel(const T* __restrict__ src, T* __restrict__ dst, long long voxels, int C, int CP) {
    long long idx = (long long)blockIdx.x * 256 + threadIdx.x;
    if (idx >= voxels * C) return;
    long long v = idx / C;
    int c = (int)(idx % C);
    dst[idx] = src[v * CP + c];
}

// up[n][s*od][s*oh][s*ow][:] = dy[n][od][oh][ow][:], zero elsewhere; up has extents (Du,Hu,Wu).
// One thread per 16 bytes of up.
__global__ void __launch_bounds__(256) spread_kernel(const uint16_t* __restrict__ dy, uint16_t* __restrict__ up, int N, int Do, int Ho,
                                                     int Wo, int Du, int Hu, int Wu, int C, int sD, int sH, int sW) {
    const int per = C / 8;
    long long total = (long long)N * Du * Hu * Wu * per;
    long long idx = (long long)blockIdx.x * 256 + threadIdx.x;
    if (idx >= total) return;
    int c8 = (int)(idx % per);
    long long v = idx / per;
    int w = (int)(v % Wu); v /= Wu;
    int h = (int)(v % Hu); v /= Hu;
    int d = (int)(v % Du);
    int n = (int)(v / Du);
    uint4 val = {0, 0, 0, 0};
    if (d % sD == 0 && h % sH == 0 && w % sW == 0) {
        int od = d / sD, oh = h / sH, ow = w / sW;
        if (od < Do && oh < Ho && ow < Wo)
            val = *(const uint4*)(dy + ((((long long)n * Do + od) * Ho + oh) * Wo + ow) * C + c8 * 8);
    }
    *(uint4*)(up + idx * 8) = val;
}

// y[n][od][oh][ow][:] = full[n][s*od][s*oh][s*ow][:]; one thread per 16 bytes of y
__global__ void __launch_bounds__(256) subsample_kernel(const uint16_t* __restrict__ full, uint16_t* __restrict__ y, int N, int Do, int Ho,
                                                        int Wo, int Du, int Hu, int Wu, int C, int sD, int sH, int sW) {
    const int per = C / 8;
    long long total = (long long)N * Do * Ho * Wo * per;
    long long idx = (long long)blockIdx.x * 256 + threadIdx.x;
    if (idx >= total) return;
    int c8 = (int)(idx % per);
    long long v = idx / per;
    int ow = (int)(v % Wo); v /= Wo;
    int oh = (int)(v % Ho); v /= Ho;
    int od = (int)(v % Do);
    int n = (int)(v / Do);
    *(uint4*)(y + idx * 8) = *(const uint4*)(full + ((((long long)n * Du + od * sD) * Hu + oh * sH) * Wu + ow * sW) * C + c8 * 8);
}

size_t align256(size_t b) { return (b + 255) & ~(size_t)255; }

unsigned blocks_for(long long n) { return (unsigned)((n + 255) / 256); }

}  // namespace

// ---- few input channels --------------------------------------------------
static Geom padded_geom(const Geom& g) {
    Geom p = g;
    p.Cin = 32;
    return p;
}

bool embed_c_supported(const Geom& g, int pass) {
    if (g.dtype != MI3D_BF16 || g.Cin >= 32) return false;
    Geom p = padded_geom(g);
    if (pass == MI3D_PASS_WGRAD) return wgrad_mfma_supported(p);
    return sp_supported(p, pass);
}

size_t embed_c_workspace_bytes(const Geom& g, int pass) {
    if (!embed_c_supported(g, pass)) return 0;
    Geom p = padded_geom(g);
    size_t xb = align256((size_t)g.in_voxels() * 32 * 2), wb = align256((size_t)p.w_elems() * 2);
    if (pass == MI3D_PASS_FWD) return xb + wb + align256(sp_workspace_bytes(p, pass));
    if (pass == MI3D_PASS_DGRAD) return xb + wb + align256(sp_workspace_bytes(p, pass));   // xb holds dx32
    return xb + align256((size_t)p.w_elems() * 4) + align256(wgrad_mfma_workspace_bytes(p));
}

int embed_c_conv(const Geom& g, int pass, const void* a, const void* b, void* out, void* ws, size_t ws_bytes, hipStream_t s) {
    if (ws_bytes < embed_c_workspace_bytes(g, pass)) return MI3D_ERR_WORKSPACE;
    Geom p = padded_geom(g);
    char* base = (char*)ws;
    const size_t xb = align256((size_t)g.in_voxels() * 32 * 2);
    uint16_t* x32 = (uint16_t*)base;
    int st;
    if (pass == MI3D_PASS_FWD || pass == MI3D_PASS_DGRAD) {
        const size_t wb = align256((size_t)p.w_elems() * 2);
        uint16_t* w32 = (uint16_t*)(base + xb);
        void* rest = base + xb + wb;
        const size_t rest_bytes = ws_bytes - xb - wb;
        const long long wrows = g.taps() * g.Cout;  // weight rows of Cin channels
        const void* w = pass == MI3D_PASS_FWD ? b : b;
        pad_channels_kernel<<<blocks_for(wrows * 4), 256, 0, s>>>((const uint16_t*)w, w32, wrows, g.Cin, 32);
        if ((st = check_launch())) return st;
        if (pass == MI3D_PASS_FWD) {
            pad_channels_kernel<<<blocks_for(g.in_voxels() * 4), 256, 0, s>>>((const uint16_t*)a, x32, g.in_voxels(), g.Cin, 32);
            if ((st = check_launch())) return st;
            return sp_conv(p, MI3D_PASS_FWD, x32, w32, out, rest, rest_bytes, s);
        }
        if ((st = sp_conv(p, MI3D_PASS_DGRAD, a, w32, x32, rest, rest_bytes, s))) return st;  // x32 = dx with 32 channels
        slice_channels_kernel<uint16_t><<<blocks_for(g.in_voxels() * g.Cin), 256, 0, s>>>(x32, (uint16_t*)out, g.in_voxels(), g.Cin, 32);
        return check_launch();
    }
    const size_t dwb = align256((size_t)p.w_elems() * 4);
    float* dw32 = (float*)(base + xb);
    void* rest = base + xb + dwb;
    pad_channels_kernel<<<blocks_for(g.in_voxels() * 4), 256, 0, s>>>((const uint16_t*)a, x32, g.in_voxels(), g.Cin, 32);
    if ((st = check_launch())) return st;
    if ((st = wgrad_mfma(p, x32, b, dw32, rest, ws_bytes - xb - dwb, s))) return st;
    const long long wrows = g.taps() * g.Cout;
    slice_channels_kernel<float><<<blocks_for(wrows * g.Cin), 256, 0, s>>>(dw32, (float*)out, wrows, g.Cin, 32);
    return check_launch();
}

// ---- stride > 1 gradients through the stride-1 kernels -------------------
static Geom unit_stride_geom(const Geom& g) {
    Geom u = g;
    u.sD = u.sH = u.sW = 1;
    u.Do = g.D + 2 * g.pD - g.kD + 1;
    u.Ho = g.H + 2 * g.pH - g.kH + 1;
    u.Wo = g.W + 2 * g.pW - g.kW + 1;
    return u;
}

bool embed_s_supported(const Geom& g, int pass) {
    if (g.dtype != MI3D_BF16 || (g.sD == 1 && g.sH == 1 && g.sW == 1)) return false;
    if (g.Cout % 8) return false;
    Geom u = unit_stride_geom(g);
    if (pass == MI3D_PASS_WGRAD) return wgrad_mfma_supported(u);
    return sp_supported(u, pass);   // forward: full-resolution output, then subsampled
}

size_t embed_s_workspace_bytes(const Geom& g, int pass) {
    if (!embed_s_supported(g, pass)) return 0;
    Geom u = unit_stride_geom(g);
    size_t up = align256((size_t)u.out_voxels() * g.Cout * 2);
    return up + align256(pass == MI3D_PASS_WGRAD ? wgrad_mfma_workspace_bytes(u) : sp_workspace_bytes(u, pass));
}

// fwd: a = x, b = w, out = y.  dgrad: a = dy, b = w, out = dx.  wgrad: a = x, b = dy, out = dw.
int embed_s_conv(const Geom& g, int pass, const void* a, const void* b, void* out, void* ws, size_t ws_bytes, hipStream_t s) {
    if (ws_bytes < embed_s_workspace_bytes(g, pass)) return MI3D_ERR_WORKSPACE;
    Geom u = unit_stride_geom(g);
    const size_t upb = align256((size_t)u.out_voxels() * g.Cout * 2);
    uint16_t* up = (uint16_t*)ws;
    void* rest = (char*)ws + upb;
    if (pass == MI3D_PASS_FWD) {  // 7/8 of the stride-1 outputs are thrown away
        int st = sp_conv(u, MI3D_PASS_FWD, a, b, up, rest, ws_bytes - upb, s);
        if (st) return st;
        subsample_kernel<<<blocks_for(g.out_voxels() * (g.Cout / 8)), 256, 0, s>>>(up, (uint16_t*)out, g.N, g.Do, g.Ho, g.Wo, u.Do, u.Ho, u.Wo,
                                                                               g.Cout, g.sD, g.sH, g.sW);
        return check_launch();
    }
    const uint16_t* dy = (const uint16_t*)(pass == MI3D_PASS_DGRAD ? a : b);
    spread_kernel<<<blocks_for(u.out_voxels() * (g.Cout / 8)), 256, 0, s>>>(dy, up, g.N, g.Do, g.Ho, g.Wo, u.Do, u.Ho, u.Wo, g.Cout,
                                                                          g.sD, g.sH, g.sW);
    int st = check_launch();
    if (st) return st;
    if (pass == MI3D_PASS_DGRAD) return sp_conv(u, MI3D_PASS_DGRAD, up, b, out, rest, ws_bytes - upb, s);
    return wgrad_mfma(u, a, up, (float*)out, rest, ws_bytes - upb, s);
}

// ---- 2x2x2 / stride 2 / pad 0 as 3x3x3 / stride 2 / pad 1 --------------------
// input index 2 o + t2 (t2 in {0,1}) == 2 o - 1 + t3 with t3 = t2 + 1: the same layer with its
// weights at taps {1,2}^3 of a 3x3x3 kernel and zeros at the 19 other taps.
namespace {
__global__ void __launch_bounds__(256) k2_to_k3_weights_kernel(const uint16_t* __restrict__ w2, uint16_t* __restrict__ w3, int Cout, int Cin) {
    long long idx = (long long)blockIdx.x * 256 + threadIdx.x;
    if (idx >= (long long)Cout * 27 * Cin) return;
    int ci = (int)(idx % Cin);
    long long r = idx / Cin;
    int t3 = (int)(r % 27);
    int co = (int)(r / 27);
    int kd = t3 / 9, kh = (t3 / 3) % 3, kw = t3 % 3;
    uint16_t v = 0;
    if (kd && kh && kw) v = w2[((long long)co * 8 + ((kd - 1) * 2 + (kh - 1)) * 2 + (kw - 1)) * Cin + ci];
    w3[idx] = v;
}
__global__ void __launch_bounds__(256) k3_to_k2_dw_kernel(const float* __restrict__ dw3, float* __restrict__ dw2, int Cout, int Cin) {
    long long idx = (long long)blockIdx.x * 256 + threadIdx.x;
    if (idx >= (long long)Cout * 8 * Cin) return;
    int ci = (int)(idx % Cin);
    long long r = idx / Cin;
    int t2 = (int)(r % 8);
    int co = (int)(r / 8);
    int t3 = ((t2 >> 2) + 1) * 9 + (((t2 >> 1) & 1) + 1) * 3 + (t2 & 1) + 1;
    dw2[idx] = dw3[((long long)co * 27 + t3) * Cin + ci];
}
Geom k3_geom(const Geom& g) {
    Geom e = g;
    e.kD = e.kH = e.kW = 3;
    e.pD = e.pH = e.pW = 1;
    return e;   // Do = (D + 2 - 3) / 2 + 1 = D / 2 for even D: unchanged
}
}  // namespace

bool embed_k2_supported(const Geom& g, int pass) {
    (void)pass;
    if (g.dtype != MI3D_BF16 || g.kD != 2 || g.kH != 2 || g.kW != 2) return false;
    if (g.sD != 2 || g.sH != 2 || g.sW != 2 || g.pD || g.pH || g.pW) return false;
    if ((g.D | g.H | g.W) & 1) return false;
    return g.Cin % 32 == 0 && g.Cout % 32 == 0;
}

size_t embed_k2_workspace_bytes(const Geom& g, int pass) {
    if (!embed_k2_supported(g, pass)) return 0;
    Geom e = k3_geom(g);
    size_t first = pass == MI3D_PASS_WGRAD ? align256((size_t)e.w_elems() * 4) : align256((size_t)e.w_elems() * 2);
    return first + align256(auto_workspace_bytes(e, pass));
}

int embed_k2_conv(const Geom& g, int pass, const void* a, const void* b, void* out, void* ws, size_t ws_bytes, hipStream_t s) {
    if (ws_bytes < embed_k2_workspace_bytes(g, pass)) return MI3D_ERR_WORKSPACE;
    Geom e = k3_geom(g);
    int st;
    if (pass == MI3D_PASS_WGRAD) {
        const size_t first = align256((size_t)e.w_elems() * 4);
        float* dw3 = (float*)ws;
        if ((st = auto_conv(e, pass, a, b, dw3, (char*)ws + first, ws_bytes - first, s))) return st;
        k3_to_k2_dw_kernel<<<blocks_for(g.w_elems()), 256, 0, s>>>(dw3, (float*)out, g.Cout, g.Cin);
        return check_launch();
    }
    const size_t first = align256((size_t)e.w_elems() * 2);
    uint16_t* w3 = (uint16_t*)ws;
    k2_to_k3_weights_kernel<<<blocks_for(e.w_elems()), 256, 0, s>>>((const uint16_t*)b, w3, g.Cout, g.Cin);
    if ((st = check_launch())) return st;
    return auto_conv(e, pass, a, w3, out, (char*)ws + first, ws_bytes - first, s);
}

}  // namespace mi3d
