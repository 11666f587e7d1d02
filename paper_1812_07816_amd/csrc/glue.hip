// Elementwise and reduction steps of the training step around the
// convolutions (network of Section 4.1): LeakyReLU, channel concatenation of
// the decoder's skip connections, sigmoid + soft Dice loss (built on the Dice
// coefficient of Section 4.3) and the SGD update.  All of them move a few
// bytes per flop, so each is one pass over its tensors with 16-byte accesses;
// reductions use a fixed partition and a fixed order (bit-reproducible).
#include <cmath>

#include "mi3d_internal.h"


namespace mi3d {
namespace {

__device__ __forceinline__ float bf16_to_f32(uint16_t v) { return __builtin_bit_cast(float, (uint32_t)v << 16); }
__device__ __forceinline__ uint16_t f32_to_bf16(float f) {  // round to nearest even; inputs are finite
    uint32_t u = __builtin_bit_cast(uint32_t, f);
    u += 0x7FFFu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}
__device__ __forceinline__ void unpack8(const uint4& v, float (&f)[8]) {
    const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        f[2 * i] = __builtin_bit_cast(float, w[i] << 16);
        f[2 * i + 1] = __builtin_bit_cast(float, w[i] & 0xFFFF0000u);
    }
}
__device__ __forceinline__ uint4 pack8(const float (&f)[8]) {
    uint32_t w[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) w[i] = (uint32_t)f32_to_bf16(f[2 * i]) | ((uint32_t)f32_to_bf16(f[2 * i + 1]) << 16);
    return uint4{w[0], w[1], w[2], w[3]};
}

// 8 consecutive values of a bf16 (F32 = false) or fp32 (F32 = true) tensor, piece index i
template <bool F32>
__device__ __forceinline__ void load8(const void* base, long long i, float (&f)[8]) {
    if (F32) {
        const float4 a = ((const float4*)base)[2 * i], b = ((const float4*)base)[2 * i + 1];
        f[0] = a.x; f[1] = a.y; f[2] = a.z; f[3] = a.w; f[4] = b.x; f[5] = b.y; f[6] = b.z; f[7] = b.w;
    } else {
        unpack8(((const uint4*)base)[i], f);
    }
}
template <bool F32>
__device__ __forceinline__ void store8(void* base, long long i, const float (&f)[8]) {
    if (F32) {
        ((float4*)base)[2 * i] = make_float4(f[0], f[1], f[2], f[3]);
        ((float4*)base)[2 * i + 1] = make_float4(f[4], f[5], f[6], f[7]);
    } else {
        ((uint4*)base)[i] = pack8(f);
    }
}

// a <- a > 0 ? a : slope * a, in place; n8 = number of 16-byte pieces
__global__ void __launch_bounds__(256) lrelu_fwd_kernel(uint4* __restrict__ a, long long n8, float slope) {
    for (long long i = (long long)blockIdx.x * 256 + threadIdx.x; i < n8; i += (long long)gridDim.x * 256) {
        float f[8];
        unpack8(a[i], f);
#pragma unroll
        for (int j = 0; j < 8; ++j) f[j] = f[j] > 0.f ? f[j] : slope * f[j];
        a[i] = pack8(f);
    }
}

// da <- da * (a > 0 ? 1 : slope), in place on da; a holds the activation's OUTPUT (same sign as its input)
template <bool F32>
__global__ void __launch_bounds__(256) lrelu_bwd_kernel(void* __restrict__ da, const void* __restrict__ a, long long n8, float slope) {
    for (long long i = (long long)blockIdx.x * 256 + threadIdx.x; i < n8; i += (long long)gridDim.x * 256) {
        float g[8], f[8];
        load8<F32>(da, i, g);
        load8<F32>(a, i, f);
#pragma unroll
        for (int j = 0; j < 8; ++j) g[j] = f[j] > 0.f ? g[j] : slope * g[j];
        store8<F32>(da, i, g);
    }
}

// out[v][0:Ca] = a[v], out[v][Ca:Ca+Cb] = b[v]; channel counts in 16-byte pieces
template <typename I>
__global__ void __launch_bounds__(256) concat_kernel(const uint4* __restrict__ a, int pa, const uint4* __restrict__ b, int pb,
                                                     uint4* __restrict__ out, I total) {
    const int pc = pa + pb;
    for (I i = (I)blockIdx.x * 256 + threadIdx.x; i < total; i += (I)gridDim.x * 256) {
        const I v = i / pc;
        const int c = (int)(i - v * pc);
        out[i] = c < pa ? a[v * pa + c] : b[v * pb + (c - pa)];
    }
}

// a[v] = in[v][0:Ca], b[v] = in[v][Ca:Ca+Cb]
template <typename I>
__global__ void __launch_bounds__(256) split_kernel(const uint4* __restrict__ in, int pa, int pb, uint4* __restrict__ a,
                                                    uint4* __restrict__ b, I total) {
    const int pc = pa + pb;
    for (I i = (I)blockIdx.x * 256 + threadIdx.x; i < total; i += (I)gridDim.x * 256) {
        const I v = i / pc;
        const int c = (int)(i - v * pc);
        const uint4 x = in[i];
        if (c < pa) a[v * pa + c] = x;
        else b[v * pb + (c - pa)] = x;
    }
}

// out[v] = in[v][off : off + C]; channel counts in 16-byte pieces
template <typename I>
__global__ void __launch_bounds__(256) slice_kernel(const uint4* __restrict__ in, int pt, int poff, int pc, uint4* __restrict__ out, I total) {
    for (I i = (I)blockIdx.x * 256 + threadIdx.x; i < total; i += (I)gridDim.x * 256) {
        const I v = i / pc;
        const int c = (int)(i - v * pc);
        out[i] = in[v * pt + poff + c];
    }
}

// out[v][off : off + C] = in[v]
template <typename I>
__global__ void __launch_bounds__(256) place_kernel(const uint4* __restrict__ in, int pc, uint4* __restrict__ out, int pt, int poff, I total) {
    for (I i = (I)blockIdx.x * 256 + threadIdx.x; i < total; i += (I)gridDim.x * 256) {
        const I v = i / pc;
        const int c = (int)(i - v * pc);
        out[v * pt + poff + c] = in[i];
    }
}

// da[v][c] <- (da[v][c] + dcat[v][off + c]) * (a[v][c] > 0 ? 1 : slope): the second gradient of a skip tensor is taken
// from its half of the concatenated tensor's gradient, and the LeakyReLU derivative of the layer that produced
// the skip tensor is applied, in one pass (fp32, one rounding)
template <typename I>
__global__ void __launch_bounds__(256) skip_grad_kernel(uint4* __restrict__ da, const uint4* __restrict__ dcat, int pt, int poff, int pc,
                                                        const uint4* __restrict__ a, I total, float slope) {
    for (I i = (I)blockIdx.x * 256 + threadIdx.x; i < total; i += (I)gridDim.x * 256) {
        const I v = i / pc;
        const int c = (int)(i - v * pc);
        float g[8], h[8], f[8];
        unpack8(da[i], g);
        unpack8(dcat[v * pt + poff + c], h);
        unpack8(a[i], f);
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const float sum = g[j] + h[j];
            g[j] = f[j] > 0.f ? sum : slope * sum;
        }
        da[i] = pack8(g);
    }
}

// a <- a + b (fp32 add, one rounding)
__global__ void __launch_bounds__(256) add_kernel(uint4* __restrict__ a, const uint4* __restrict__ b, long long n8) {
    for (long long i = (long long)blockIdx.x * 256 + threadIdx.x; i < n8; i += (long long)gridDim.x * 256) {
        float f[8], g[8];
        unpack8(a[i], f);
        unpack8(b[i], g);
#pragma unroll
        for (int j = 0; j < 8; ++j) f[j] += g[j];
        a[i] = pack8(f);
    }
}

__device__ __forceinline__ float sigmoidf(float x) { return 1.f / (1.f + __expf(-x)); }

// Soft Dice, first pass.  A thread takes groups of 8 voxels = 8 C values (C 16-byte pieces of logits, C 8-byte
// pieces of labels); value e of a group belongs to class e % C.  Per class: sum p t, sum p, sum t.  A block
// owns a contiguous range of groups; per-thread sums are combined in a fixed tree and written as one partial.
template <int C, bool F32>
__global__ void __launch_bounds__(256) dice_partial_kernel(const void* __restrict__ logits, const uint2* __restrict__ labels,
                                                           long long groups, float* __restrict__ part) {
    __shared__ float red[3 * C][256];
    const long long g0 = groups * blockIdx.x / gridDim.x, g1 = groups * (blockIdx.x + 1) / gridDim.x;
    float s[3 * C];
#pragma unroll
    for (int k = 0; k < 3 * C; ++k) s[k] = 0.f;
    for (long long g = g0 + threadIdx.x; g < g1; g += 256) {
#pragma unroll
        for (int q = 0; q < C; ++q) {
            float x[8];
            load8<F32>(logits, g * C + q, x);
            const uint2 lb = labels[g * C + q];
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const int cls = (8 * q + j) % C;
                const float t = (float)(((j < 4 ? lb.x : lb.y) >> (8 * (j & 3))) & 0xFFu);
                const float p = sigmoidf(x[j]);
                s[cls] += p * t;
                s[C + cls] += p;
                s[2 * C + cls] += t;
            }
        }
    }
#pragma unroll
    for (int k = 0; k < 3 * C; ++k) red[k][threadIdx.x] = s[k];
    __syncthreads();
    for (int w = 128; w > 0; w >>= 1) {
        if (threadIdx.x < w) {
#pragma unroll
            for (int k = 0; k < 3 * C; ++k) red[k][threadIdx.x] += red[k][threadIdx.x + w];
        }
        __syncthreads();
    }
    if (threadIdx.x < 3 * C) part[blockIdx.x * 3 * C + threadIdx.x] = red[threadIdx.x][0];
}

// second pass: thread t adds partials t, t + 256, ... in double, then a fixed binary tree over the threads
// (bit-reproducible); sums[3C] and the loss 1 - mean_c (2 I + eps) / (P + T + eps)
template <int C>
__global__ void __launch_bounds__(256) dice_final_kernel(const float* __restrict__ part, int nblocks, float eps, float* __restrict__ sums, float* __restrict__ loss) {
    __shared__ double red[3 * C][256];
    const int t = threadIdx.x;
    double a[3 * C];
#pragma unroll
    for (int q = 0; q < 3 * C; ++q) a[q] = 0.0;
    for (int b = t; b < nblocks; b += 256)
#pragma unroll
        for (int q = 0; q < 3 * C; ++q) a[q] += (double)part[b * 3 * C + q];
#pragma unroll
    for (int q = 0; q < 3 * C; ++q) red[q][t] = a[q];
    __syncthreads();
    for (int s = 128; s > 0; s >>= 1) {
        if (t < s)
#pragma unroll
            for (int q = 0; q < 3 * C; ++q) red[q][t] += red[q][t + s];
        __syncthreads();
    }
    if (t < 3 * C) sums[t] = (float)red[t][0];
    if (t == 0) {
        double d = 0.0;
        for (int c = 0; c < C; ++c) d += (2.0 * red[c][0] + eps) / (red[C + c][0] + red[2 * C + c][0] + eps);
        *loss = (float)(1.0 - d / C);
    }
}

// dloss/dlogit = -(1/C) (2 t den - (2 I + eps)) / den^2 * p (1 - p), den = P + T + eps
template <int C, bool F32>
__global__ void __launch_bounds__(256) dice_grad_kernel(const void* __restrict__ logits, const uint2* __restrict__ labels, long long groups,
                                                        float eps, const float* __restrict__ sums, void* __restrict__ dlogits) {
    float ka[C], kb[C];  // gradient wrt p = ka * t + kb
#pragma unroll
    for (int c = 0; c < C; ++c) {
        const float den = sums[C + c] + sums[2 * C + c] + eps;
        ka[c] = -2.f / (den * C);
        kb[c] = (2.f * sums[c] + eps) / (den * den * C);
    }
    for (long long g = (long long)blockIdx.x * 256 + threadIdx.x; g < groups; g += (long long)gridDim.x * 256) {
#pragma unroll
        for (int q = 0; q < C; ++q) {
            float x[8];
            load8<F32>(logits, g * C + q, x);
            const uint2 lb = labels[g * C + q];
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const int cls = (8 * q + j) % C;
                const float t = (float)(((j < 4 ? lb.x : lb.y) >> (8 * (j & 3))) & 0xFFu);
                const float p = sigmoidf(x[j]);
                x[j] = (ka[cls] * t + kb[cls]) * p * (1.f - p);
            }
            store8<F32>(dlogits, g * C + q, x);
        }
    }
}

// w <- w - lr * dw (fp32 master weights), wb <- bf16(w)
__global__ void __launch_bounds__(256) sgd_kernel(float* __restrict__ w, const float* __restrict__ dw, uint16_t* __restrict__ wb, long long n, float lr) {
    for (long long i = (long long)blockIdx.x * 256 + threadIdx.x; i < n; i += (long long)gridDim.x * 256) {
        const float v = w[i] - lr * dw[i];
        w[i] = v;
        if (wb) wb[i] = f32_to_bf16(v);
    }
}

// Adam (the optimiser of Section 4.1) on fp32 state: m <- b1 m + (1 - b1) g, v <- b2 v + (1 - b2) g^2,
// w <- w - lr (m / c1) / (sqrt(v / c2) + eps) with the bias corrections c1 = 1 - b1^t, c2 = 1 - b2^t; wb <- bf16(w)
__global__ void __launch_bounds__(256) adam_kernel(float* __restrict__ w, const float* __restrict__ dw, float* __restrict__ m, float* __restrict__ v,
                                                   uint16_t* __restrict__ wb, long long n, float lr, float b1, float b2, float eps, float c1, float c2) {
    for (long long i = (long long)blockIdx.x * 256 + threadIdx.x; i < n; i += (long long)gridDim.x * 256) {
        const float g = dw[i];
        const float mi = b1 * m[i] + (1.f - b1) * g;
        const float vi = b2 * v[i] + (1.f - b2) * g * g;
        m[i] = mi;
        v[i] = vi;
        const float x = w[i] - lr * (mi / c1) / (sqrtf(vi / c2) + eps);
        w[i] = x;
        if (wb) wb[i] = f32_to_bf16(x);
    }
}

unsigned grid_for(long long items) {
    long long b = (items + 255) / 256;
    return (unsigned)(b < 1 ? 1 : (b > 8192 ? 8192 : b));
}
bool al16(const void* p) { return ((uintptr_t)p & 15) == 0; }
constexpr int DICE_BLOCKS = 1024;

}  // namespace
}  // namespace mi3d

using namespace mi3d;

extern "C" {

int mi3d_leaky_relu_fwd(void* a, size_t n, float slope, void* stream) {
    if (!a || !al16(a) || n % 8) return MI3D_ERR_INVALID_ARG;
    if (n == 0) return MI3D_OK;
    lrelu_fwd_kernel<<<grid_for(n / 8), 256, 0, (hipStream_t)stream>>>((uint4*)a, (long long)(n / 8), slope);
    return check_launch();
}

int mi3d_leaky_relu_bwd(void* da, const void* a, size_t n, float slope, void* stream) {
    if (!da || !a || !al16(da) || !al16(a) || n % 8) return MI3D_ERR_INVALID_ARG;
    if (n == 0) return MI3D_OK;
    lrelu_bwd_kernel<false><<<grid_for(n / 8), 256, 0, (hipStream_t)stream>>>(da, a, (long long)(n / 8), slope);
    return check_launch();
}

int mi3d_leaky_relu_bwd_f32(float* da, const float* a, size_t n, float slope, void* stream) {
    if (!da || !a || !al16(da) || !al16(a) || n % 8) return MI3D_ERR_INVALID_ARG;
    if (n == 0) return MI3D_OK;
    lrelu_bwd_kernel<true><<<grid_for(n / 8), 256, 0, (hipStream_t)stream>>>(da, a, (long long)(n / 8), slope);
    return check_launch();
}

int mi3d_concat_channels(const void* a, int Ca, const void* b, int Cb, void* out, size_t voxels, void* stream) {
    if (!a || !b || !out || !al16(a) || !al16(b) || !al16(out) || Ca <= 0 || Cb <= 0 || Ca % 8 || Cb % 8) return MI3D_ERR_INVALID_ARG;
    if (voxels == 0) return MI3D_OK;
    const long long total = (long long)voxels * ((Ca + Cb) / 8);
    if (total < (1ll << 31)) concat_kernel<unsigned><<<grid_for(total), 256, 0, (hipStream_t)stream>>>((const uint4*)a, Ca / 8, (const uint4*)b, Cb / 8, (uint4*)out, (unsigned)total);
    else concat_kernel<long long><<<grid_for(total), 256, 0, (hipStream_t)stream>>>((const uint4*)a, Ca / 8, (const uint4*)b, Cb / 8, (uint4*)out, total);
    return check_launch();
}

int mi3d_split_channels(const void* in, int Ca, int Cb, void* a, void* b, size_t voxels, void* stream) {
    if (!a || !b || !in || !al16(a) || !al16(b) || !al16(in) || Ca <= 0 || Cb <= 0 || Ca % 8 || Cb % 8) return MI3D_ERR_INVALID_ARG;
    if (voxels == 0) return MI3D_OK;
    const long long total = (long long)voxels * ((Ca + Cb) / 8);
    if (total < (1ll << 31)) split_kernel<unsigned><<<grid_for(total), 256, 0, (hipStream_t)stream>>>((const uint4*)in, Ca / 8, Cb / 8, (uint4*)a, (uint4*)b, (unsigned)total);
    else split_kernel<long long><<<grid_for(total), 256, 0, (hipStream_t)stream>>>((const uint4*)in, Ca / 8, Cb / 8, (uint4*)a, (uint4*)b, total);
    return check_launch();
}

int mi3d_slice_channels(const void* in, int C_total, int c_off, int C, void* out, size_t voxels, void* stream) {
    if (!in || !out || !al16(in) || !al16(out) || C <= 0 || c_off < 0 || c_off + C > C_total || C % 8 || c_off % 8 || C_total % 8) return MI3D_ERR_INVALID_ARG;
    if (voxels == 0) return MI3D_OK;
    const long long total = (long long)voxels * (C / 8);
    if ((long long)voxels * (C_total / 8) < (1ll << 31)) slice_kernel<unsigned><<<grid_for(total), 256, 0, (hipStream_t)stream>>>((const uint4*)in, C_total / 8, c_off / 8, C / 8, (uint4*)out, (unsigned)total);
    else slice_kernel<long long><<<grid_for(total), 256, 0, (hipStream_t)stream>>>((const uint4*)in, C_total / 8, c_off / 8, C / 8, (uint4*)out, total);
    return check_launch();
}

int mi3d_place_channels(const void* in, int C, void* out, int C_total, int c_off, size_t voxels, void* stream) {
    if (!in || !out || !al16(in) || !al16(out) || C <= 0 || c_off < 0 || c_off + C > C_total || C % 8 || c_off % 8 || C_total % 8) return MI3D_ERR_INVALID_ARG;
    if (voxels == 0) return MI3D_OK;
    const long long total = (long long)voxels * (C / 8);
    if ((long long)voxels * (C_total / 8) < (1ll << 31)) place_kernel<unsigned><<<grid_for(total), 256, 0, (hipStream_t)stream>>>((const uint4*)in, C / 8, (uint4*)out, C_total / 8, c_off / 8, (unsigned)total);
    else place_kernel<long long><<<grid_for(total), 256, 0, (hipStream_t)stream>>>((const uint4*)in, C / 8, (uint4*)out, C_total / 8, c_off / 8, total);
    return check_launch();
}

int mi3d_skip_grad(void* da, const void* dcat, int C_total, int c_off, const void* a, int C, size_t voxels, float slope, void* stream) {
    if (!da || !dcat || !a || !al16(da) || !al16(dcat) || !al16(a)) return MI3D_ERR_INVALID_ARG;
    if (C <= 0 || c_off < 0 || c_off + C > C_total || C % 8 || c_off % 8 || C_total % 8) return MI3D_ERR_INVALID_ARG;
    if (voxels == 0) return MI3D_OK;
    const long long total = (long long)voxels * (C / 8);
    if ((long long)voxels * (C_total / 8) < (1ll << 31)) skip_grad_kernel<unsigned><<<grid_for(total), 256, 0, (hipStream_t)stream>>>((uint4*)da, (const uint4*)dcat, C_total / 8, c_off / 8, C / 8, (const uint4*)a, (unsigned)total, slope);
    else skip_grad_kernel<long long><<<grid_for(total), 256, 0, (hipStream_t)stream>>>((uint4*)da, (const uint4*)dcat, C_total / 8, c_off / 8, C / 8, (const uint4*)a, total, slope);
    return check_launch();
}

int mi3d_add_inplace(void* a, const void* b, size_t n, void* stream) {
    if (!a || !b || !al16(a) || !al16(b) || n % 8) return MI3D_ERR_INVALID_ARG;
    if (n == 0) return MI3D_OK;
    add_kernel<<<grid_for(n / 8), 256, 0, (hipStream_t)stream>>>((uint4*)a, (const uint4*)b, (long long)(n / 8));
    return check_launch();
}

size_t mi3d_dice_workspace_bytes(int classes) { return (size_t)DICE_BLOCKS * 3 * (classes > 0 ? classes : 1) * sizeof(float); }

static int dice_loss_any(bool f32, const void* logits, const uint8_t* labels, size_t voxels, int classes, float eps,
                         void* ws, size_t ws_bytes, float* sums, float* loss, void* stream) {
    if (!logits || !labels || !ws || !sums || !loss || !al16(logits) || ((uintptr_t)labels & 7) || voxels == 0 || voxels % 8) return MI3D_ERR_INVALID_ARG;
    if (classes != 3) return MI3D_ERR_UNSUPPORTED;
    if (ws_bytes < mi3d_dice_workspace_bytes(classes)) return MI3D_ERR_WORKSPACE;
    const long long groups = (long long)(voxels / 8);
    const int blocks = (int)(groups < DICE_BLOCKS ? groups : DICE_BLOCKS);
    if (f32) dice_partial_kernel<3, true><<<blocks, 256, 0, (hipStream_t)stream>>>(logits, (const uint2*)labels, groups, (float*)ws);
    else dice_partial_kernel<3, false><<<blocks, 256, 0, (hipStream_t)stream>>>(logits, (const uint2*)labels, groups, (float*)ws);
    int st = check_launch();
    if (st) return st;
    dice_final_kernel<3><<<1, 256, 0, (hipStream_t)stream>>>((const float*)ws, blocks, eps, sums, loss);
    return check_launch();
}

static int dice_grad_any(bool f32, const void* logits, const uint8_t* labels, size_t voxels, int classes, float eps,
                         const float* sums, void* dlogits, void* stream) {
    if (!logits || !labels || !sums || !dlogits || !al16(logits) || !al16(dlogits) || ((uintptr_t)labels & 7) || voxels == 0 || voxels % 8)
        return MI3D_ERR_INVALID_ARG;
    if (classes != 3) return MI3D_ERR_UNSUPPORTED;
    const long long groups = (long long)(voxels / 8);
    if (f32) dice_grad_kernel<3, true><<<grid_for(groups), 256, 0, (hipStream_t)stream>>>(logits, (const uint2*)labels, groups, eps, sums, dlogits);
    else dice_grad_kernel<3, false><<<grid_for(groups), 256, 0, (hipStream_t)stream>>>(logits, (const uint2*)labels, groups, eps, sums, dlogits);
    return check_launch();
}

int mi3d_dice_loss(const void* logits, const uint8_t* labels, size_t voxels, int classes, float eps,
                   void* ws, size_t ws_bytes, float* sums, float* loss, void* stream) {
    return dice_loss_any(false, logits, labels, voxels, classes, eps, ws, ws_bytes, sums, loss, stream);
}

int mi3d_dice_grad(const void* logits, const uint8_t* labels, size_t voxels, int classes, float eps,
                   const float* sums, void* dlogits, void* stream) {
    return dice_grad_any(false, logits, labels, voxels, classes, eps, sums, dlogits, stream);
}

int mi3d_dice_loss_f32(const float* logits, const uint8_t* labels, size_t voxels, int classes, float eps,
                       void* ws, size_t ws_bytes, float* sums, float* loss, void* stream) {
    return dice_loss_any(true, logits, labels, voxels, classes, eps, ws, ws_bytes, sums, loss, stream);
}

int mi3d_dice_grad_f32(const float* logits, const uint8_t* labels, size_t voxels, int classes, float eps,
                       const float* sums, float* dlogits, void* stream) {
    return dice_grad_any(true, logits, labels, voxels, classes, eps, sums, dlogits, stream);
}

int mi3d_sgd_update(float* w, const float* dw, void* w_bf16, size_t n, float lr, void* stream) {
    if (!w || !dw) return MI3D_ERR_INVALID_ARG;
    if (n == 0) return MI3D_OK;
    sgd_kernel<<<grid_for((long long)n), 256, 0, (hipStream_t)stream>>>(w, dw, (uint16_t*)w_bf16, (long long)n, lr);
    return check_launch();
}

int mi3d_adam_update(float* w, const float* dw, float* m, float* v, void* w_bf16, size_t n, float lr, float beta1, float beta2, float eps,
                     int step, void* stream) {
    if (!w || !dw || !m || !v || step < 1) return MI3D_ERR_INVALID_ARG;
    if (!(beta1 >= 0.f && beta1 < 1.f && beta2 >= 0.f && beta2 < 1.f && eps > 0.f)) return MI3D_ERR_INVALID_ARG;
    if (n == 0) return MI3D_OK;
    const float c1 = (float)(1.0 - pow((double)beta1, (double)step)), c2 = (float)(1.0 - pow((double)beta2, (double)step));
    adam_kernel<<<grid_for((long long)n), 256, 0, (hipStream_t)stream>>>(w, dw, m, v, (uint16_t*)w_bf16, (long long)n, lr, beta1, beta2, eps, c1, c2);
    return check_launch();
}

}  // extern "C"
