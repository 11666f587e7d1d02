// Internal declarations shared by the translation units of libmi3d.so.
#pragma once
#include <hip/hip_runtime.h>
#include <atomic>
#include <stddef.h>
#include <stdint.h>

#include "../../include/mi3d.h"

namespace mi3d {

// Validated geometry of one layer (descriptor plus derived output extents).
struct Geom {
    int N, D, H, W, Cin;
    int Cout, kD, kH, kW;
    int sD, sH, sW, pD, pH, pW;
    int Do, Ho, Wo;
    int dtype;
    // Optional fused epilogue, set by the dispatcher only for kernels that implement it.  Forward: LeakyReLU with
    // `slope` on the output.  Data gradient: dx is multiplied by (ref > 0 ? 1 : slope), the LeakyReLU derivative of
    // the layer below, whose activated output `ref` has the shape of dx.
    float slope = 1.f;
    const void* ref = nullptr;
    // Optional channel-range view of the tensor of x's shape (x of the forward pass and the weight gradient, dx of
    // the data gradient): it lives in a tensor with x_pitch channels per voxel, starting at channel x_off
    // (x_pitch = 0: dense).  Set by the dispatcher only for kernels that implement it.
    int x_pitch = 0, x_off = 0;
    // Optional virtual concatenation: the tensor of x's shape is given as two tensors of Cin / 2 channels each, the
    // pointer of the call being the low half and `hi` the high half.  Set by the dispatcher only for kernels that
    // implement it.
    const void* hi = nullptr;
    // Optional second gradient of dx's shape added to the bf16-rounded data gradient before the factor of `ref` /
    // `slope` is applied (skip connection).  Set by the dispatcher only for kernels that implement it.
    const void* add = nullptr;
    // Optional statistics of the forward output for the instance normalisation that follows: stats[n][c] =
    // (mean, 1 / sqrt(var + stats_eps)) over the voxels.  In a data-gradient pass: the two means the backward pass of
    // the instance normalisation of the layer below needs, (mean g, mean g xhat) with g = dx lrelu'(ref) and
    // xhat = lrelu^-1(ref) (slope = the LeakyReLU's).  Set by the dispatcher only for kernels that implement it.
    float* stats = nullptr;
    float stats_eps = 0.f;
    __host__ __device__ long long in_voxels() const { return (long long)N * D * H * W; }
    __host__ __device__ long long out_voxels() const { return (long long)N * Do * Ho * Wo; }
    __host__ __device__ long long taps() const { return (long long)kD * kH * kW; }
    __host__ __device__ long long w_elems() const { return taps() * Cin * Cout; }
    // One D-plane of either activation tensor stays below 2 GiB in bf16: the tiled kernels address inside a plane
    // with 32-bit offsets (the plane base is a 64-bit pointer).
    bool planes_fit_32bit() const {
        return (long long)H * W * (x_pitch ? x_pitch : Cin) * 2 < (1ll << 31) && (long long)Ho * Wo * Cout * 2 < (1ll << 31);
    }
    __host__ __device__ size_t esize() const { return dtype == MI3D_BF16 ? 2 : 4; }
};

int make_geom(const mi3d_conv_desc* d, Geom* g);  // MI3D_OK or error
void note_hip_error(hipError_t e);
int check_launch();  // hipGetLastError -> status

// bf16 helpers (device): storage is the upper 16 bits of the fp32 pattern.
__device__ __forceinline__ float bf16_to_f32(uint16_t v) { return __uint_as_float((uint32_t)v << 16); }
__device__ __forceinline__ uint16_t f32_to_bf16_rne(float f) {
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return 0x7fc0;  // NaN stays NaN
    u += 0x7fffu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

// ---- kernel families (each returns a status; only enqueue on `stream`) ----
// plain one-thread-per-output kernels: any geometry, both dtypes
size_t direct_workspace_bytes(const Geom& g, int pass);
int direct_fwd(const Geom& g, const void* x, const void* w, void* y, hipStream_t s);
int direct_dgrad(const Geom& g, const void* dy, const void* w, void* dx, hipStream_t s);
int direct_wgrad(const Geom& g, const void* x, const void* dy, float* dw, void* ws, size_t ws_bytes, hipStream_t s);
// y[i] = bf16(act(sum_c part[c * n + i])), chunks added in index order; n8 = n / 8 outputs of 8; act = LeakyReLU with
// `slope` (ref null) or the factor (ref[i] > 0 ? 1 : slope).  y_hi non-null: the output, `cout` channels per voxel, is
// written as two tensors of cout / 2 channels per voxel (y the low half, y_hi the high half); cout / 2 % 8 == 0.
// add non-null (with ref): the sum is rounded to bf16, add[i] is added and the factor applied, then rounded again.
__global__ void sum_chunks_bf16_kernel(const float* __restrict__ part, uint16_t* __restrict__ y, long long n8, long long n, int nch,
                                       float slope, const uint16_t* __restrict__ ref, uint16_t* __restrict__ y_hi, int cout,
                                       const uint16_t* __restrict__ add);
// out[i] = sum_p part[p*n + i] in a fixed order (bit-reproducible); launch with (n + 15) / 16 blocks of 256
__global__ void reduce_partials_kernel(const float* __restrict__ part, float* __restrict__ out, long long n, int parts);
// out[i] = sum_p part[p * n + i] in an order fixed by (n, parts); picks the kernel by the number of parts
int reduce_partials(const float* part, float* out, long long n, int parts, hipStream_t s);


// plane-streaming MFMA kernel: bf16, 3x3x3, stride 1 (forward and data gradient)
bool sp_supported(const Geom& g, int pass);
size_t sp_workspace_bytes(const Geom& g, int pass);
int sp_conv(const Geom& g, int pass, const void* in, const void* w, void* out, void* ws, size_t ws_bytes, hipStream_t s);
bool sp_fuses_dgrad_factor(const Geom& g);  // the forward LeakyReLU is always fused
bool sp_fuses_stats(const Geom& g);         // instance-normalisation statistics of the forward output
bool sp_fuses_bwd_sums(const Geom& g);      // sums of the instance-normalisation backward pass from the data gradient
int sp_stats_finish(const float* part, const int* key, int Cout, int CT, int N, int nwg, int max_seg, double inv_v, float eps, int means,
                    float* stats, hipStream_t s);   // statistics (or plain means) from partial sums in the plane-streaming kernel's layout
bool dgrad_s2_fuses_skip_sums(const Geom& g);       // stride-2 data gradient with added gradient and the normalisation's backward sums
bool c4_fwd_fuses_stats(const Geom& g);     // the first layer's forward kernel delivers them too
// last step of a per-(sample, channel) reduction of two quantities: means from block sums part[n][block][2][C]
int instnorm_finish_means(const float* part, int blocks, int C, int N, double inv_v, float* out, hipStream_t s);


// MFMA weight gradient: bf16, 3x3x3, stride 1, channels in multiples of 32
bool wgrad_mfma_supported(const Geom& g);
size_t wgrad_mfma_workspace_bytes(const Geom& g);
int wgrad_mfma(const Geom& g, const void* x, const void* dy, float* dw, void* ws, size_t ws_bytes, hipStream_t s);


// MFMA forward pass of the 3x3x3 stride-2 convolution with 32 input channels
bool s2_fwd_supported(const Geom& g);
size_t s2_fwd_workspace_bytes(const Geom& g);
int s2_fwd(const Geom& g, const void* x, const void* w, void* y, void* ws, size_t ws_bytes, hipStream_t s);


// fallbacks through the stride-1 MFMA kernels: zero-padded input channels, zero-spread dy
bool embed_c_supported(const Geom& g, int pass);
size_t embed_c_workspace_bytes(const Geom& g, int pass);
int embed_c_conv(const Geom& g, int pass, const void* a, const void* b, void* out, void* ws, size_t ws_bytes, hipStream_t s);
bool embed_s_supported(const Geom& g, int pass);
size_t embed_s_workspace_bytes(const Geom& g, int pass);
int embed_s_conv(const Geom& g, int pass, const void* a, const void* b, void* out, void* ws, size_t ws_bytes, hipStream_t s);


// MFMA weight gradient of the 3x3x3 stride-2 convolution, channels in multiples of 32
bool wgrad_s2_supported(const Geom& g);
size_t wgrad_s2_workspace_bytes(const Geom& g);
int wgrad_s2(const Geom& g, const void* x, const void* dy, float* dw, void* ws, size_t ws_bytes, hipStream_t s);


// 2x2x2 stride-2 pad-0 layers (decoder up-sampling): forward (gather) and data gradient (scatter) as panel GEMMs
bool k2_supported(const Geom& g, int pass);
size_t k2_workspace_bytes(const Geom& g, int pass);
int k2_conv(const Geom& g, int pass, const void* a, const void* w, void* out, void* ws, size_t ws_bytes, hipStream_t s);
// first-layer kernels (4 input channels)
bool c4_fwd_supported(const Geom& g);
size_t c4_fwd_workspace_bytes(const Geom& g);
int c4_fwd(const Geom& g, const void* x, const void* w, void* y, void* ws, size_t ws_bytes, hipStream_t s);
bool c4_dgrad_supported(const Geom& g);
size_t c4_dgrad_workspace_bytes(const Geom& g);
int c4_dgrad(const Geom& g, const void* dy, const void* w, void* dx, void* ws, size_t ws_bytes, hipStream_t s);
bool c4_wgrad_supported(const Geom& g);
size_t c4_wgrad_workspace_bytes(const Geom& g);
int c4_wgrad(const Geom& g, const void* x, const void* dy, float* dw, void* ws, size_t ws_bytes, hipStream_t s);


// MFMA data gradient of the 3x3x3 stride-2 convolution (equal pads 0/1, Cout 32 or 64)
bool dgrad_s2_supported(const Geom& g);
size_t dgrad_s2_workspace_bytes(const Geom& g);
int dgrad_s2(const Geom& g, const void* dy, const void* w, void* dx, void* ws, size_t ws_bytes, hipStream_t s);
bool dgrad_s2_fuses_factor(const Geom& g);
bool dgrad_s2_fuses_skip(const Geom& g);   // the added second gradient of a skip connection


// 1x1x1 convolution to <= 4 output channels (segmentation head), all passes
bool pointwise_supported(const Geom& g);
size_t pointwise_workspace_bytes(const Geom& g, int pass);
int pointwise_conv(const Geom& g, int pass, const void* a, const void* b, void* out, void* ws, size_t ws_bytes, hipStream_t s);
// the same head in fp32 (VALU kernels; the fp32 dispatcher routes 1x1x1 layers with at most 4 output channels here)
bool pointwise_f32_supported(const Geom& g);
size_t pointwise_f32_workspace_bytes(const Geom& g, int pass);
int pointwise_f32_conv(const Geom& g, int pass, const void* a, const void* b, void* out, void* ws, size_t ws_bytes, hipStream_t s);


// 2x2x2 stride-2 pad-0 layers (decoder upsampling and its gradients) run as 3x3x3 stride-2 pad-1 layers
// whose weights sit at taps {1,2}^3 (even extents only)
bool embed_k2_supported(const Geom& g, int pass);
size_t embed_k2_workspace_bytes(const Geom& g, int pass);
int embed_k2_conv(const Geom& g, int pass, const void* a, const void* b, void* out, void* ws, size_t ws_bytes, hipStream_t s);

// fp32 MFMA kernels: any kernel extent up to 3 and stride up to 2 (forward, data gradient, weight gradient)
bool f32_supported(const Geom& g, int pass);
size_t f32_workspace_bytes(const Geom& g, int pass);
int f32_conv(const Geom& g, int pass, const void* in, const void* w, void* out, void* ws, size_t ws_bytes, hipStream_t s);
int f32_wgrad(const Geom& g, const void* x, const void* dy, float* dw, void* ws, size_t ws_bytes, hipStream_t s);
bool f32_wgrad_folds_taps(const Geom& g);   // at most 4 input channels: (tap, channel) pairs as the columns of the MFMA block
bool f32_takes_halves(const Geom& g, int pass);   // the tensor of x's shape as two halves along the channels

// automatic kernel choice for a geometry (a, b, out per pass: fwd (x, w, y), dgrad (dy, w, dx), wgrad (x, dy, dw))
size_t auto_workspace_bytes(const Geom& g, int pass);
int auto_conv(const Geom& g, int pass, const void* a, const void* b, void* out, void* ws, size_t ws_bytes, hipStream_t s);

}  // namespace mi3d
