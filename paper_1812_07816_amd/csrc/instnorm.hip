// Instance normalisation of the network of Section 4.1 (each convolution is followed by an instance
// normalisation and a LeakyReLU), without learnable scale and shift:
//   xhat[n,v,c] = (z[n,v,c] - mean[n,c]) * rstd[n,c],   mean / var over the voxels v of one sample and channel,
//   rstd = 1 / sqrt(var + eps) (biased variance),        a = lrelu(xhat).
// Only the activated tensor a is kept for the backward pass: LeakyReLU with a positive slope is invertible, so
// xhat = a > 0 ? a : a / slope is taken back from it, and the statistics (N x C x 2 floats) ride along.  Backward:
//   g = da * lrelu'(xhat),   dz = rstd * (g - mean_v(g) - xhat * mean_v(g * xhat)).
// All four steps stream NDHWC tensors once with 16-byte accesses (bf16, or fp32 in the entry points named _f32:
// the same kernels on 32-byte pieces); the two reductions use a fixed partition of the voxels into blocks and add
// the block sums in index order in double (bit-reproducible).
#include "mi3d_internal.h"

namespace mi3d {
namespace {

constexpr int IN_BLOCKS = 512;   // voxel ranges per sample
constexpr int MAXC = 512;

__device__ __forceinline__ void unpack8(const uint4& v, float (&f)[8]) {
    const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        f[2 * i] = __builtin_bit_cast(float, w[i] << 16);
        f[2 * i + 1] = __builtin_bit_cast(float, w[i] & 0xFFFF0000u);
    }
}
__device__ __forceinline__ uint4 pack8(const float (&f)[8]) {
    typedef __attribute__((__vector_size__(2 * sizeof(float)))) float f32x2;
    typedef __attribute__((__vector_size__(2 * sizeof(__bf16)))) __bf16 bf16x2;
    uint32_t w[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        f32x2 p = {f[2 * i], f[2 * i + 1]};
        w[i] = __builtin_bit_cast(uint32_t, __builtin_convertvector(p, bf16x2));
    }
    return uint4{w[0], w[1], w[2], w[3]};
}

// A piece = the 8 channels a thread handles at a time: one 16-byte word of bf16, or two of fp32.
struct Raw32 { float4 lo, hi; };
template <typename T> struct Piece;
template <> struct Piece<uint16_t> {
    typedef uint4 raw;
    static __device__ __forceinline__ void unpack(const raw& v, float (&f)[8]) { unpack8(v, f); }
    static __device__ __forceinline__ raw pack(const float (&f)[8]) { return pack8(f); }
};
template <> struct Piece<float> {
    typedef Raw32 raw;
    static __device__ __forceinline__ void unpack(const raw& v, float (&f)[8]) {
        f[0] = v.lo.x; f[1] = v.lo.y; f[2] = v.lo.z; f[3] = v.lo.w; f[4] = v.hi.x; f[5] = v.hi.y; f[6] = v.hi.z; f[7] = v.hi.w;
    }
    static __device__ __forceinline__ raw pack(const float (&f)[8]) {
        return Raw32{float4{f[0], f[1], f[2], f[3]}, float4{f[4], f[5], f[6], f[7]}};
    }
};

// Sums of two quantities per channel over the voxel range of block (blockIdx.x, sample blockIdx.y).
// MODE 0: (z, z^2) of one tensor.  MODE 1: (g, g * xhat) with g = da * lrelu'(xhat), xhat from a.
// Thread t handles the 8 channels of piece t % P of voxels t / P, t / P + VPB, ...; the per-thread sums of a piece
// are added over the voxel lanes in lane order.  part: [n][block][2][C].
template <int MODE, typename T>
__global__ void __launch_bounds__(256) in_reduce_kernel(const T* __restrict__ a, const T* __restrict__ da, long long voxels, int C,
                                                        float slope, float* __restrict__ part) {
    typedef typename Piece<T>::raw raw;
    __shared__ float red[256 * 8];
    const int P = C / 8, VPB = 256 / P;         // pieces per voxel, voxels per pass of the block
    const int t = threadIdx.x, p = t % P, lane = t / P;
    const int n = blockIdx.y;
    const long long v0 = voxels * blockIdx.x / gridDim.x, v1 = voxels * (blockIdx.x + 1) / gridDim.x;
    float s1[8], s2[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) s1[j] = s2[j] = 0.f;
    const float inv_slope = 1.f / slope;
    // one voxel's contribution; the loop below requests four voxels ahead of the arithmetic (the sums are added in
    // voxel order either way)
    auto add_voxel = [&](const raw& av, const raw& gv) {
        float x[8];
        Piece<T>::unpack(av, x);
        if (MODE == 0) {
#pragma unroll
            for (int j = 0; j < 8; ++j) { s1[j] += x[j]; s2[j] = fmaf(x[j], x[j], s2[j]); }
        } else {
            float g[8];
            Piece<T>::unpack(gv, g);
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const float gg = x[j] > 0.f ? g[j] : slope * g[j];
                const float xh = x[j] > 0.f ? x[j] : x[j] * inv_slope;
                s1[j] += gg;
                s2[j] = fmaf(gg, xh, s2[j]);
            }
        }
    };
    if (lane < VPB) {
        const long long base = (long long)n * voxels * C + p * 8;
        long long v = v0 + lane;
        for (; v + 3 * VPB < v1; v += 4 * VPB) {
            raw av[4], gv[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                av[u] = *(const raw*)(a + base + (v + u * VPB) * C);
                gv[u] = MODE == 0 ? av[u] : *(const raw*)(da + base + (v + u * VPB) * C);
            }
#pragma unroll
            for (int u = 0; u < 4; ++u) add_voxel(av[u], gv[u]);
        }
        for (; v < v1; v += VPB) {
            const raw av = *(const raw*)(a + base + v * C);
            add_voxel(av, MODE == 0 ? av : *(const raw*)(da + base + v * C));
        }
    }
    float* out = part + ((long long)n * gridDim.x + blockIdx.x) * 2 * C;
    for (int q = 0; q < 2; ++q) {
        __syncthreads();
#pragma unroll
        for (int j = 0; j < 8; ++j) red[t * 8 + j] = lane < VPB ? (q ? s2[j] : s1[j]) : 0.f;
        __syncthreads();
        for (int c = t; c < C; c += 256) {
            const int pp = c / 8, j = c % 8;
            float s = 0.f;
            for (int l = 0; l < VPB; ++l) s += red[(l * P + pp) * 8 + j];
            out[q * C + c] = s;
        }
    }
}

// MODE 0: stats[n][c] = (mean, rstd) from the block sums of (z, z^2).  MODE 1: stats2[n][c] = (mean g, mean g xhat).
// A workgroup serves 16 (n, c) pairs; thread (slice s, pair i) adds blocks s, s + 16, ... in double and the 16 slice
// sums are added in order (bit-reproducible).
template <int MODE>
__global__ void __launch_bounds__(256) in_finish_kernel(const float* __restrict__ part, int blocks, int C, int total, double inv_v, float eps,
                                                        float* __restrict__ out) {
    __shared__ double r1[16][17], r2[16][17];
    const int il = threadIdx.x & 15, sl = threadIdx.x >> 4;
    const int i = blockIdx.x * 16 + il;     // (n, c)
    double s1 = 0.0, s2 = 0.0;
    if (i < total) {
        const int n = i / C, c = i - n * C;
        for (int b = sl; b < blocks; b += 16) {
            const float* pb = part + ((long long)n * blocks + b) * 2 * C;
            s1 += (double)pb[c];
            s2 += (double)pb[C + c];
        }
    }
    r1[sl][il] = s1; r2[sl][il] = s2;
    __syncthreads();
    if (sl != 0 || i >= total) return;
    s1 = 0.0; s2 = 0.0;
    for (int k = 0; k < 16; ++k) { s1 += r1[k][il]; s2 += r2[k][il]; }
    if (MODE == 0) {
        const double mean = s1 * inv_v;
        double var = s2 * inv_v - mean * mean;
        if (var < 0.0) var = 0.0;
        out[2 * i] = (float)mean;
        out[2 * i + 1] = (float)(1.0 / sqrt(var + (double)eps));
    } else {
        out[2 * i] = (float)(s1 * inv_v);
        out[2 * i + 1] = (float)(s2 * inv_v);
    }
}

// a <- lrelu((z - mean) * rstd), in place.  One sample per blockIdx.y; its statistics sit in LDS.
template <typename T>
__global__ void __launch_bounds__(256) in_fwd_kernel(typename Piece<T>::raw* __restrict__ z, const float* __restrict__ stats, long long pieces, int C,
                                                     float slope) {
    typedef typename Piece<T>::raw raw;
    __shared__ float st[2 * MAXC];
    const int n = blockIdx.y, P = C / 8;
    for (int i = threadIdx.x; i < 2 * C; i += 256) st[i] = stats[(long long)n * 2 * C + i];
    __syncthreads();
    raw* zn = z + (long long)n * pieces;
    const long long i0 = (long long)blockIdx.x * 256 + threadIdx.x;
    int pc = (int)(i0 % P);                                  // piece within the voxel, advanced without a division
    const int pstep = (int)(((long long)gridDim.x * 256) % P);
    for (long long i = i0; i < pieces; i += (long long)gridDim.x * 256, pc = pc + pstep >= P ? pc + pstep - P : pc + pstep) {
        const int c0 = pc * 8;
        float x[8];
        Piece<T>::unpack(zn[i], x);
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const float xh = (x[j] - st[2 * (c0 + j)]) * st[2 * (c0 + j) + 1];
            x[j] = fmaxf(xh, slope * xh);
        }
        zn[i] = Piece<T>::pack(x);
    }
}

// da <- dz = rstd * (g - mean g - xhat * mean(g xhat)), in place; st: (mean, rstd), s2: (mean g, mean g xhat)
template <typename T>
__global__ void __launch_bounds__(256) in_bwd_kernel(typename Piece<T>::raw* __restrict__ da, const typename Piece<T>::raw* __restrict__ a,
                                                     const float* __restrict__ stats, const float* __restrict__ sums, long long pieces, int C,
                                                     float slope) {
    typedef typename Piece<T>::raw raw;
    __shared__ float rs[MAXC], m1[MAXC], m2[MAXC];
    const int n = blockIdx.y, P = C / 8;
    for (int i = threadIdx.x; i < C; i += 256) {
        rs[i] = stats[((long long)n * C + i) * 2 + 1];
        m1[i] = sums[((long long)n * C + i) * 2];
        m2[i] = sums[((long long)n * C + i) * 2 + 1];
    }
    __syncthreads();
    raw* dn = da + (long long)n * pieces;
    const raw* an = a + (long long)n * pieces;
    const float inv_slope = 1.f / slope;
    const long long i0 = (long long)blockIdx.x * 256 + threadIdx.x;
    int pc = (int)(i0 % P);
    const int pstep = (int)(((long long)gridDim.x * 256) % P);
    for (long long i = i0; i < pieces; i += (long long)gridDim.x * 256, pc = pc + pstep >= P ? pc + pstep - P : pc + pstep) {
        const int c0 = pc * 8;
        float g[8], x[8];
        Piece<T>::unpack(dn[i], g);
        Piece<T>::unpack(an[i], x);
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const float gg = x[j] > 0.f ? g[j] : slope * g[j];
            const float xh = x[j] > 0.f ? x[j] : x[j] * inv_slope;
            g[j] = rs[c0 + j] * (gg - m1[c0 + j] - xh * m2[c0 + j]);
        }
        dn[i] = Piece<T>::pack(g);
    }
}

bool in_args_ok(int N, size_t voxels, int C) {
    return N > 0 && voxels > 0 && C > 0 && C % 8 == 0 && C <= MAXC && N <= 65535;
}
int in_blocks(size_t voxels) { return (int)(voxels < (size_t)IN_BLOCKS ? voxels : (size_t)IN_BLOCKS); }
unsigned in_grid(long long pieces) {
    long long b = (pieces + 255) / 256;
    return (unsigned)(b < 1 ? 1 : (b > 4096 ? 4096 : b));
}
bool a16(const void* p) { return ((uintptr_t)p & 15) == 0; }

}  // namespace

// out[n][c] = (mean of the first quantity, mean of the second) from block sums part[n][block][2][C], added in index order
// in double: the last step of a reduction whose block sums another kernel has written in in_reduce_kernel's layout
int instnorm_finish_means(const float* part, int blocks, int C, int N, double inv_v, float* out, hipStream_t s) {
    in_finish_kernel<1><<<(N * C + 15) / 16, 256, 0, s>>>(part, blocks, C, N * C, inv_v, 0.f, out);
    return check_launch();
}

namespace {

template <typename T>
int in_stats(const void* z, int N, size_t voxels, int C, float eps, float* stats, void* ws, size_t ws_bytes, void* stream) {
    if (!z || !stats || !ws || !a16(z) || !in_args_ok(N, voxels, C) || !(eps > 0.f)) return MI3D_ERR_INVALID_ARG;
    if (ws_bytes < mi3d_instnorm_workspace_bytes(N, C)) return MI3D_ERR_WORKSPACE;
    const int blocks = in_blocks(voxels);
    in_reduce_kernel<0, T><<<dim3(blocks, N), 256, 0, (hipStream_t)stream>>>((const T*)z, nullptr, (long long)voxels, C, 1.f, (float*)ws);
    int st = check_launch();
    if (st) return st;
    in_finish_kernel<0><<<(N * C + 15) / 16, 256, 0, (hipStream_t)stream>>>((const float*)ws, blocks, C, N * C, 1.0 / (double)voxels, eps, stats);
    return check_launch();
}

template <typename T>
int in_fwd(void* z, const float* stats, int N, size_t voxels, int C, float slope, void* stream) {
    typedef typename Piece<T>::raw raw;
    if (!z || !stats || !a16(z) || !in_args_ok(N, voxels, C) || !(slope > 0.f && slope <= 1.f)) return MI3D_ERR_INVALID_ARG;
    const long long pieces = (long long)voxels * (C / 8);
    in_fwd_kernel<T><<<dim3(in_grid(pieces), N), 256, 0, (hipStream_t)stream>>>((raw*)z, stats, pieces, C, slope);
    return check_launch();
}

template <typename T>
int in_bwd(void* da, const void* a, const float* stats, int N, size_t voxels, int C, float slope, void* ws, size_t ws_bytes, void* stream) {
    typedef typename Piece<T>::raw raw;
    if (!da || !a || !stats || !ws || !a16(da) || !a16(a) || !in_args_ok(N, voxels, C) || !(slope > 0.f && slope <= 1.f)) return MI3D_ERR_INVALID_ARG;
    if (ws_bytes < mi3d_instnorm_workspace_bytes(N, C)) return MI3D_ERR_WORKSPACE;
    const int blocks = in_blocks(voxels);
    float* part = (float*)ws;
    float* sums = part + (size_t)N * IN_BLOCKS * 2 * C;
    in_reduce_kernel<1, T><<<dim3(blocks, N), 256, 0, (hipStream_t)stream>>>((const T*)a, (const T*)da, (long long)voxels, C, slope, part);
    int st = check_launch();
    if (st) return st;
    in_finish_kernel<1><<<(N * C + 15) / 16, 256, 0, (hipStream_t)stream>>>(part, blocks, C, N * C, 1.0 / (double)voxels, 0.f, sums);
    if ((st = check_launch())) return st;
    const long long pieces = (long long)voxels * (C / 8);
    in_bwd_kernel<T><<<dim3(in_grid(pieces), N), 256, 0, (hipStream_t)stream>>>((raw*)da, (const raw*)a, stats, sums, pieces, C, slope);
    return check_launch();
}

}  // namespace

}  // namespace mi3d

using namespace mi3d;

extern "C" {

size_t mi3d_instnorm_workspace_bytes(int N, int C) {
    if (N <= 0 || C <= 0) return 0;
    return ((size_t)N * IN_BLOCKS * 2 * C + (size_t)N * C * 2) * sizeof(float);
}

int mi3d_instnorm_stats(const void* z, int N, size_t voxels, int C, float eps, float* stats, void* ws, size_t ws_bytes, void* stream) {
    return in_stats<uint16_t>(z, N, voxels, C, eps, stats, ws, ws_bytes, stream);
}
int mi3d_instnorm_stats_f32(const void* z, int N, size_t voxels, int C, float eps, float* stats, void* ws, size_t ws_bytes, void* stream) {
    return in_stats<float>(z, N, voxels, C, eps, stats, ws, ws_bytes, stream);
}

int mi3d_instnorm_lrelu_fwd(void* z, const float* stats, int N, size_t voxels, int C, float slope, void* stream) {
    return in_fwd<uint16_t>(z, stats, N, voxels, C, slope, stream);
}
int mi3d_instnorm_lrelu_fwd_f32(void* z, const float* stats, int N, size_t voxels, int C, float slope, void* stream) {
    return in_fwd<float>(z, stats, N, voxels, C, slope, stream);
}

int mi3d_instnorm_lrelu_bwd(void* da, const void* a, const float* stats, int N, size_t voxels, int C, float slope, void* ws, size_t ws_bytes,
                            void* stream) {
    return in_bwd<uint16_t>(da, a, stats, N, voxels, C, slope, ws, ws_bytes, stream);
}
int mi3d_instnorm_lrelu_bwd_f32(void* da, const void* a, const float* stats, int N, size_t voxels, int C, float slope, void* ws, size_t ws_bytes,
                                void* stream) {
    return in_bwd<float>(da, a, stats, N, voxels, C, slope, ws, ws_bytes, stream);
}

int mi3d_instnorm_lrelu_bwd_sums(void* da, const void* a, const float* stats, const float* sums, int N, size_t voxels, int C, float slope,
                                 void* stream) {
    if (!da || !a || !stats || !sums || !a16(da) || !a16(a) || !in_args_ok(N, voxels, C) || !(slope > 0.f && slope <= 1.f)) return MI3D_ERR_INVALID_ARG;
    const long long pieces = (long long)voxels * (C / 8);
    in_bwd_kernel<uint16_t><<<dim3(in_grid(pieces), N), 256, 0, (hipStream_t)stream>>>((uint4*)da, (const uint4*)a, stats, sums, pieces, C, slope);
    return check_launch();
}

}  // extern "C"
