// 1x1x1 convolution to a handful of output channels (the segmentation head:
// 32 -> 3 classes).  All three passes are bound by streaming the 32-channel
// tensor once (3 flop/byte), so they are plain vector-ALU kernels built around
// 16-byte loads and stores:
//   fwd    y[v,co]  = sum_ci x[v,ci] w[co,ci]      a thread per 8 input channels of a voxel, lanes of a voxel summed
//   dgrad  dx[v,ci] = sum_co dy[v,co] w[co,ci]     a thread per 8 input channels of a voxel, grid-stride
//   wgrad  dw[co,ci]= sum_v dy[v,co] x[v,ci]       per-thread partial sums over a strided voxel range,
//                                                  block tree reduction, slots added in fixed order
// Supported: k = 1, s = 1, p = 0, Cin % 8 == 0, Cin <= 64, Cout <= 4, bf16.
#include "mi3d_internal.h"

namespace mi3d {
namespace {

constexpr int MAXCI = 64, MAXCO = 4;

__device__ __forceinline__ void unpack8(const uint4& v, float (&f)[8]) {
    const uint32_t u[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        f[2 * i] = __uint_as_float(u[i] << 16);
        f[2 * i + 1] = __uint_as_float(u[i] & 0xffff0000u);
    }
}

// Thread t of the grid handles the 16-byte pieces t, t + T, ... of x (8 input channels of one voxel), four at a time;
// the Cin / 8 neighbouring lanes that share a voxel add their partial sums in a fixed butterfly and the first of
// them stores the voxel's outputs.
template <int CO>
__global__ void __launch_bounds__(256) pw_fwd_kernel(const uint16_t* __restrict__ x, const uint16_t* __restrict__ w,
                                                     uint16_t* __restrict__ y, long long voxels, int Cin) {
    __shared__ float ws[MAXCO * MAXCI];
    for (int i = threadIdx.x; i < CO * Cin; i += 256) ws[i] = bf16_to_f32(w[i]);
    __syncthreads();
    const int per = Cin / 8;                      // a power of two that divides 64: a voxel never straddles waves
    const long long pieces = voxels * per, T = (long long)gridDim.x * 256;
    const int c0 = (threadIdx.x % per) * 8;       // T is a multiple of per: the same channels in every round
    constexpr int U = 4;
    for (long long i0 = (long long)blockIdx.x * 256 + threadIdx.x; i0 < pieces; i0 += U * T) {   // (uniform over the lanes of a voxel)
        uint4 xv[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const long long i = i0 + u * T;
            xv[u] = *(const uint4*)(x + (i < pieces ? i : pieces - 1) * 8);   // clamped: loaded, never stored
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const long long i = i0 + u * T;
            float f[8], acc[CO];
            unpack8(xv[u], f);
#pragma unroll
            for (int co = 0; co < CO; ++co) {
                acc[co] = 0.f;
#pragma unroll
                for (int j = 0; j < 8; ++j) acc[co] = fmaf(f[j], ws[co * Cin + c0 + j], acc[co]);
            }
            for (int off = per >> 1; off > 0; off >>= 1)
#pragma unroll
                for (int co = 0; co < CO; ++co) acc[co] += __shfl_xor(acc[co], off, 64);
            if (c0 == 0 && i < pieces) {
                const long long v = i / per;
#pragma unroll
                for (int co = 0; co < CO; ++co) y[v * CO + co] = f32_to_bf16_rne(acc[co]);
            }
        }
    }
}

// Thread t of the grid handles the 16-byte pieces t, t + T, t + 2 T, ... of dx (T = threads in the grid), four at a time
// so that their loads are in flight together; a piece is 8 input channels of one voxel.
// SUMS: one sample per blockIdx.y; no factor is applied to dx, but with a = ref (the activated output of the
// normalised layer below), g = dx * lrelu'(a) of the stored values and xhat = lrelu^-1(a), every thread adds up g and
// g * xhat of its 8 channels (T is a multiple of the pieces per voxel, so they are the same in every round); the block
// adds its threads' sums in thread order and writes part[n][block][2][Cin].
template <int CO, bool SUMS>
__global__ void __launch_bounds__(256) pw_dgrad_kernel(const uint16_t* __restrict__ dy, const uint16_t* __restrict__ w,
                                                       uint16_t* __restrict__ dx, long long voxels, int Cin,
                                                       const uint16_t* __restrict__ ref, float slope, float* __restrict__ part) {
    __shared__ float ws[MAXCO * MAXCI];
    __shared__ float red[SUMS ? 256 * 8 : 1];
    for (int i = threadIdx.x; i < CO * Cin; i += 256) ws[i] = bf16_to_f32(w[i]);
    __syncthreads();
    const int per = Cin / 8;
    if (SUMS) {   // this block's sample
        dy += (long long)blockIdx.y * voxels * CO;
        dx += (long long)blockIdx.y * voxels * Cin;
        ref += (long long)blockIdx.y * voxels * Cin;
    }
    const long long pieces = voxels * per, T = (long long)gridDim.x * 256;
    constexpr int U = 4;
    float s1[8], s2[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) s1[j] = s2[j] = 0.f;
    const float inv_slope = 1.f / slope;
    for (long long i0 = (long long)blockIdx.x * 256 + threadIdx.x; i0 < pieces; i0 += U * T) {
        float g[U][CO];
        uint4 m4[U];
        long long idx[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            idx[u] = i0 + u * T;
            const long long ic = idx[u] < pieces ? idx[u] : pieces - 1;   // clamped: loaded, never stored
            const long long v = ic / per;
#pragma unroll
            for (int co = 0; co < CO; ++co) g[u][co] = bf16_to_f32(dy[v * CO + co]);
            // optional LeakyReLU derivative of the layer below: factor 1 where its activated output ref is > 0, slope elsewhere
            m4[u] = uint4{0x3f803f80u, 0x3f803f80u, 0x3f803f80u, 0x3f803f80u};
            if (ref) m4[u] = *(const uint4*)(ref + ic * 8);
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            if (idx[u] >= pieces) continue;
            const int c0 = (int)(idx[u] % per) * 8;
            const uint32_t m[4] = {m4[u].x, m4[u].y, m4[u].z, m4[u].w};
            uint32_t o[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                float a = 0.f, b = 0.f;
#pragma unroll
                for (int co = 0; co < CO; ++co) {
                    a = fmaf(g[u][co], ws[co * Cin + c0 + 2 * j], a);
                    b = fmaf(g[u][co], ws[co * Cin + c0 + 2 * j + 1], b);
                }
                if (!SUMS) {
                    if (!((int)(m[j] << 16) > 0)) a *= slope;
                    if (!((int)(m[j] & 0xffff0000u) > 0)) b *= slope;
                }
                o[j] = (uint32_t)f32_to_bf16_rne(a) | ((uint32_t)f32_to_bf16_rne(b) << 16);
                if (SUMS) {
                    const float va = __uint_as_float(o[j] << 16), vb = __uint_as_float(o[j] & 0xffff0000u);
                    const float ra = __uint_as_float(m[j] << 16), rb = __uint_as_float(m[j] & 0xffff0000u);
                    const float ga = ra > 0.f ? va : slope * va, gb = rb > 0.f ? vb : slope * vb;
                    s1[2 * j] += ga; s2[2 * j] = fmaf(ga, ra > 0.f ? ra : ra * inv_slope, s2[2 * j]);
                    s1[2 * j + 1] += gb; s2[2 * j + 1] = fmaf(gb, rb > 0.f ? rb : rb * inv_slope, s2[2 * j + 1]);
                }
            }
            *(uint4*)(dx + idx[u] * 8) = uint4{o[0], o[1], o[2], o[3]};
        }
    }
    if (SUMS) {
        const int t = threadIdx.x, groups = 256 / per;    // thread t holds channels 8 (t % per) ..
        float* out = part + ((long long)blockIdx.y * gridDim.x + blockIdx.x) * 2 * Cin;
        for (int q = 0; q < 2; ++q) {
            __syncthreads();
#pragma unroll
            for (int j = 0; j < 8; ++j) red[t * 8 + j] = q ? s2[j] : s1[j];
            __syncthreads();
            for (int c = t; c < Cin; c += 256) {
                const int pp = c / 8, j = c % 8;
                float a = 0.f;
                for (int l = 0; l < groups; ++l) a += red[(l * per + pp) * 8 + j];
                out[q * Cin + c] = a;
            }
        }
    }
}

// block b handles voxels b, b + gridDim.x, ... in chunks; thread (g = t / per, c8 = t % per): voxel lane g
template <int CO>
__global__ void __launch_bounds__(256) pw_wgrad_kernel(const uint16_t* __restrict__ x, const uint16_t* __restrict__ dy,
                                                       float* __restrict__ part, long long voxels, int Cin) {
    __shared__ float red[256 * 8];
    const int per = Cin / 8, groups = 256 / per;
    const int t = threadIdx.x, g = t / per, c8 = t % per;
    float acc[CO][8];
#pragma unroll
    for (int co = 0; co < CO; ++co)
#pragma unroll
        for (int j = 0; j < 8; ++j) acc[co][j] = 0.f;
    if (g < groups)
        for (long long v = (long long)blockIdx.x * groups + g; v < voxels; v += (long long)gridDim.x * groups) {
            float f[8];
            unpack8(*(const uint4*)(x + v * Cin + c8 * 8), f);
#pragma unroll
            for (int co = 0; co < CO; ++co) {
                const float gv = bf16_to_f32(dy[v * CO + co]);
#pragma unroll
                for (int j = 0; j < 8; ++j) acc[co][j] = fmaf(gv, f[j], acc[co][j]);
            }
        }
    // fixed-order reduction over the voxel lanes g of the block, one cout at a time
    for (int co = 0; co < CO; ++co) {
        __syncthreads();
#pragma unroll
        for (int j = 0; j < 8; ++j) red[t * 8 + j] = (g < groups) ? acc[co][j] : 0.f;
        __syncthreads();
        if (t < Cin) {
            const int cc8 = t / 8, j = t % 8;
            float a = 0.f;
            for (int gg = 0; gg < groups; ++gg) a += red[(gg * per + cc8) * 8 + j];
            part[((long long)blockIdx.x * CO + co) * Cin + t] = a;
        }
    }
}

// ---- the same three passes for fp32 tensors (a piece is 8 channels = 32 bytes, two 16-byte accesses; a thread keeps
//      the same channels throughout, so its weights stay in registers) ------------------------------------------------
__device__ __forceinline__ void load8f(const float* p, float (&f)[8]) {
    const float4 a = *(const float4*)p, b = *(const float4*)(p + 4);
    f[0] = a.x; f[1] = a.y; f[2] = a.z; f[3] = a.w; f[4] = b.x; f[5] = b.y; f[6] = b.z; f[7] = b.w;
}

// y = lrelu(x . w) (slope 1: none); lanes of a voxel summed in a fixed butterfly
template <int CO>
__global__ void __launch_bounds__(256) pwf_fwd_kernel(const float* __restrict__ x, const float* __restrict__ w, float* __restrict__ y,
                                                      long long voxels, int Cin, float slope) {
    const int per = Cin / 8;
    const long long pieces = voxels * per, T = (long long)gridDim.x * 256;
    const int c0 = (threadIdx.x % per) * 8;
    float wr[CO][8];
#pragma unroll
    for (int co = 0; co < CO; ++co) load8f(w + co * Cin + c0, wr[co]);
    constexpr int U = 4;
    for (long long i0 = (long long)blockIdx.x * 256 + threadIdx.x; i0 < pieces; i0 += U * T) {   // (uniform over the lanes of a voxel)
        float f[U][8];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const long long i = i0 + u * T;
            load8f(x + (i < pieces ? i : pieces - 1) * 8, f[u]);   // clamped: loaded, never stored
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const long long i = i0 + u * T;
            float acc[CO];
#pragma unroll
            for (int co = 0; co < CO; ++co) {
                acc[co] = 0.f;
#pragma unroll
                for (int j = 0; j < 8; ++j) acc[co] = fmaf(f[u][j], wr[co][j], acc[co]);
            }
            for (int off = per >> 1; off > 0; off >>= 1)
#pragma unroll
                for (int co = 0; co < CO; ++co) acc[co] += __shfl_xor(acc[co], off, 64);
            if (c0 == 0 && i < pieces) {
                const long long v = i / per;
#pragma unroll
                for (int co = 0; co < CO; ++co) y[v * CO + co] = fmaxf(acc[co], slope * acc[co]);
            }
        }
    }
}

// dx = (dy . w^T) * (ref > 0 ? 1 : slope) (no ref: no factor)
template <int CO>
__global__ void __launch_bounds__(256) pwf_dgrad_kernel(const float* __restrict__ dy, const float* __restrict__ w, float* __restrict__ dx,
                                                        long long voxels, int Cin, const float* __restrict__ ref, float slope) {
    const int per = Cin / 8;
    const long long pieces = voxels * per, T = (long long)gridDim.x * 256;
    const int c0 = (threadIdx.x % per) * 8;
    float wr[CO][8];
#pragma unroll
    for (int co = 0; co < CO; ++co) load8f(w + co * Cin + c0, wr[co]);
    constexpr int U = 4;
    for (long long i0 = (long long)blockIdx.x * 256 + threadIdx.x; i0 < pieces; i0 += U * T) {
        float g[U][CO], m[U][8];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const long long i = i0 + u * T, ic = i < pieces ? i : pieces - 1;
            const long long v = ic / per;
#pragma unroll
            for (int co = 0; co < CO; ++co) g[u][co] = dy[v * CO + co];
#pragma unroll
            for (int j = 0; j < 8; ++j) m[u][j] = 1.f;
            if (ref) load8f(ref + ic * 8, m[u]);
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const long long i = i0 + u * T;
            if (i >= pieces) continue;
            float o[8];
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                float a = 0.f;
#pragma unroll
                for (int co = 0; co < CO; ++co) a = fmaf(g[u][co], wr[co][j], a);
                o[j] = m[u][j] > 0.f ? a : slope * a;
            }
            *(float4*)(dx + i * 8) = make_float4(o[0], o[1], o[2], o[3]);
            *(float4*)(dx + i * 8 + 4) = make_float4(o[4], o[5], o[6], o[7]);
        }
    }
}

// per-block partial sums of dw over a strided voxel range, as pw_wgrad_kernel
template <int CO>
__global__ void __launch_bounds__(256) pwf_wgrad_kernel(const float* __restrict__ x, const float* __restrict__ dy, float* __restrict__ part,
                                                        long long voxels, int Cin) {
    __shared__ float red[256 * 8];
    const int per = Cin / 8, groups = 256 / per;
    const int t = threadIdx.x, g = t / per, c8 = t % per;
    float acc[CO][8];
#pragma unroll
    for (int co = 0; co < CO; ++co)
#pragma unroll
        for (int j = 0; j < 8; ++j) acc[co][j] = 0.f;
    const long long V = (long long)gridDim.x * groups;
    constexpr int U = 2;
    for (long long v0 = (long long)blockIdx.x * groups + g; v0 < voxels; v0 += U * V) {
        float f[U][8], gv[U][CO];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const long long v = v0 + u * V, vc = v < voxels ? v : voxels - 1;
            load8f(x + vc * Cin + c8 * 8, f[u]);
#pragma unroll
            for (int co = 0; co < CO; ++co) gv[u][co] = v < voxels ? dy[vc * CO + co] : 0.f;   // past the end: adds zeros
        }
#pragma unroll
        for (int u = 0; u < U; ++u)
#pragma unroll
            for (int co = 0; co < CO; ++co)
#pragma unroll
                for (int j = 0; j < 8; ++j) acc[co][j] = fmaf(gv[u][co], f[u][j], acc[co][j]);
    }
    for (int co = 0; co < CO; ++co) {
        __syncthreads();
#pragma unroll
        for (int j = 0; j < 8; ++j) red[t * 8 + j] = acc[co][j];
        __syncthreads();
        if (t < Cin) {
            const int cc8 = t / 8, j = t % 8;
            float a = 0.f;
            for (int gg = 0; gg < groups; ++gg) a += red[(gg * per + cc8) * 8 + j];
            part[((long long)blockIdx.x * CO + co) * Cin + t] = a;
        }
    }
}

}  // namespace

bool pointwise_supported(const Geom& g) {
    if (g.dtype != MI3D_BF16 || g.kD != 1 || g.kH != 1 || g.kW != 1) return false;
    if (g.sD != 1 || g.sH != 1 || g.sW != 1 || g.pD || g.pH || g.pW) return false;
    return g.Cin % 8 == 0 && g.Cin <= MAXCI && g.Cout <= MAXCO && 256 % (g.Cin / 8) == 0;
}

static int pw_wgrad_blocks(const Geom& g) {
    long long groups = 256 / (g.Cin / 8);
    long long b = (g.in_voxels() + groups - 1) / groups;
    return (int)(b < 1024 ? b : 1024);
}

constexpr int PW_SUM_BLOCKS = 512;   // blocks per sample of the data gradient that also adds up the normalisation's sums

size_t pointwise_workspace_bytes(const Geom& g, int pass) {
    if (!pointwise_supported(g) || pass == MI3D_PASS_FWD) return 0;
    if (pass == MI3D_PASS_DGRAD) return (size_t)g.N * PW_SUM_BLOCKS * 2 * g.Cin * sizeof(float);   // block sums of the variant with sums
    return (size_t)pw_wgrad_blocks(g) * g.Cout * g.Cin * sizeof(float);
}

template <int CO>
static int pw_run(const Geom& g, int pass, const void* a, const void* b, void* out, void* ws, hipStream_t s) {
    const long long vox = g.in_voxels();
    if (pass == MI3D_PASS_FWD) {
        long long blocks = (vox * (g.Cin / 8) + 4 * 256 - 1) / (4 * 256);
        if (blocks > 8192) blocks = 8192;
        pw_fwd_kernel<CO><<<(unsigned)blocks, 256, 0, s>>>((const uint16_t*)a, (const uint16_t*)b, (uint16_t*)out, vox, g.Cin);
        return check_launch();
    }
    if (pass == MI3D_PASS_DGRAD && g.stats) {
        // with the two sums of the instance-normalisation backward pass of the layer below (ref = its activated output)
        if (!g.ref || !(g.slope > 0.f) || g.N > 65535) return MI3D_ERR_UNSUPPORTED;
        const long long per_sample = vox / g.N;
        long long blocks = (per_sample * (g.Cin / 8) + 4 * 256 - 1) / (4 * 256);
        if (blocks > PW_SUM_BLOCKS) blocks = PW_SUM_BLOCKS;
        pw_dgrad_kernel<CO, true><<<dim3((unsigned)blocks, (unsigned)g.N), 256, 0, s>>>((const uint16_t*)a, (const uint16_t*)b, (uint16_t*)out, per_sample,
                                                                                        g.Cin, (const uint16_t*)g.ref, g.slope, (float*)ws);
        int st = check_launch();
        if (st) return st;
        return instnorm_finish_means((const float*)ws, (int)blocks, g.Cin, g.N, 1.0 / (double)per_sample, g.stats, s);
    }
    if (pass == MI3D_PASS_DGRAD) {
        const long long n = vox * (g.Cin / 8);
        long long blocks = (n + 4 * 256 - 1) / (4 * 256);
        if (blocks > 8192) blocks = 8192;
        pw_dgrad_kernel<CO, false><<<(unsigned)blocks, 256, 0, s>>>((const uint16_t*)a, (const uint16_t*)b, (uint16_t*)out, vox, g.Cin,
                                                                     (const uint16_t*)g.ref, g.slope, nullptr);
        return check_launch();
    }
    const int blocks = pw_wgrad_blocks(g);
    pw_wgrad_kernel<CO><<<blocks, 256, 0, s>>>((const uint16_t*)a, (const uint16_t*)b, (float*)ws, vox, g.Cin);
    int st = check_launch();
    if (st) return st;
    const long long n = (long long)g.Cout * g.Cin;
    return reduce_partials((const float*)ws, (float*)out, n, blocks, s);
}

static int pwf_wgrad_blocks(const Geom& g) {
    long long groups = 256 / (g.Cin / 8);
    long long b = (g.in_voxels() + groups - 1) / groups;
    return (int)(b < 2048 ? b : 2048);
}

bool pointwise_f32_supported(const Geom& g) {
    if (g.dtype != MI3D_F32 || g.kD != 1 || g.kH != 1 || g.kW != 1) return false;
    if (g.sD != 1 || g.sH != 1 || g.sW != 1 || g.pD || g.pH || g.pW) return false;
    // (lanes of a voxel must share a wave: Cin/8 a power of two)
    return g.Cin % 8 == 0 && g.Cin <= MAXCI && g.Cout <= MAXCO && 64 % (g.Cin / 8) == 0 && g.in_voxels() * (g.Cin / 8) / 256 <= 0x7fffffffll;
}

size_t pointwise_f32_workspace_bytes(const Geom& g, int pass) {
    if (!pointwise_f32_supported(g) || pass != MI3D_PASS_WGRAD) return 0;
    return (size_t)pwf_wgrad_blocks(g) * g.Cout * g.Cin * sizeof(float);
}

template <int CO>
static int pwf_run(const Geom& g, int pass, const void* a, const void* b, void* out, void* ws, hipStream_t s) {
    const long long vox = g.in_voxels();
    long long blocks = (vox * (g.Cin / 8) + 4 * 256 - 1) / (4 * 256);
    if (blocks > 8192) blocks = 8192;
    if (pass == MI3D_PASS_FWD) {
        pwf_fwd_kernel<CO><<<(unsigned)blocks, 256, 0, s>>>((const float*)a, (const float*)b, (float*)out, vox, g.Cin, g.slope);
        return check_launch();
    }
    if (pass == MI3D_PASS_DGRAD) {
        pwf_dgrad_kernel<CO><<<(unsigned)blocks, 256, 0, s>>>((const float*)a, (const float*)b, (float*)out, vox, g.Cin, (const float*)g.ref, g.slope);
        return check_launch();
    }
    const int nb = pwf_wgrad_blocks(g);
    pwf_wgrad_kernel<CO><<<nb, 256, 0, s>>>((const float*)a, (const float*)b, (float*)ws, vox, g.Cin);
    int st = check_launch();
    if (st) return st;
    return reduce_partials((const float*)ws, (float*)out, (long long)g.Cout * g.Cin, nb, s);
}

// the fp32 head: same arguments as pointwise_conv; applies the optional LeakyReLU (forward) or derivative factor (data gradient)
int pointwise_f32_conv(const Geom& g, int pass, const void* a, const void* b, void* out, void* ws, size_t ws_bytes, hipStream_t s) {
    if (!pointwise_f32_supported(g) || g.add || g.hi) return MI3D_ERR_UNSUPPORTED;
    if (ws_bytes < pointwise_f32_workspace_bytes(g, pass)) return MI3D_ERR_WORKSPACE;
    switch (g.Cout) {
        case 1: return pwf_run<1>(g, pass, a, b, out, ws, s);
        case 2: return pwf_run<2>(g, pass, a, b, out, ws, s);
        case 3: return pwf_run<3>(g, pass, a, b, out, ws, s);
        default: return pwf_run<4>(g, pass, a, b, out, ws, s);
    }
}

// fwd: a = x, b = w, out = y.  dgrad: a = dy, b = w, out = dx.  wgrad: a = x, b = dy, out = dw.
int pointwise_conv(const Geom& g, int pass, const void* a, const void* b, void* out, void* ws, size_t ws_bytes, hipStream_t s) {
    if (ws_bytes < pointwise_workspace_bytes(g, pass)) return MI3D_ERR_WORKSPACE;
    if (g.in_voxels() * (g.Cin / 8) / 256 > 0x7fffffffll) return MI3D_ERR_UNSUPPORTED;
    switch (g.Cout) {
        case 1: return pw_run<1>(g, pass, a, b, out, ws, s);
        case 2: return pw_run<2>(g, pass, a, b, out, ws, s);
        case 3: return pw_run<3>(g, pass, a, b, out, ws, s);
        default: return pw_run<4>(g, pass, a, b, out, ws, s);
    }
}

}  // namespace mi3d
