// Plain convolution kernels: one thread per output element, any geometry,
// fp32 or bf16 storage with fp32 accumulation.  They are the fallback for
// shapes no tuned kernel covers and a slow cross-check for the MFMA kernels.
// Definitions: forward / data-gradient / weight-gradient of the feature-map
// layers whose outputs are kept for the backward pass (Section 3.1).
#include "mi3d_internal.h"

namespace mi3d {
namespace {

template <typename T> struct Elem;
template <> struct Elem<float> {
    static __device__ __forceinline__ float load(const float* p) { return *p; }
    static __device__ __forceinline__ void store(float* p, float v) { *p = v; }
};
template <> struct Elem<uint16_t> {
    static __device__ __forceinline__ float load(const uint16_t* p) { return bf16_to_f32(*p); }
    static __device__ __forceinline__ void store(uint16_t* p, float v) { *p = f32_to_bf16_rne(v); }
};

template <typename T>
__global__ void __launch_bounds__(256) fwd_kernel(Geom g, const T* __restrict__ x, const T* __restrict__ w, T* __restrict__ y) {
    long long total = g.out_voxels() * g.Cout;
    long long idx = (long long)blockIdx.x * 256 + threadIdx.x;
    if (idx >= total) return;
    int co = (int)(idx % g.Cout);
    long long v = idx / g.Cout;
    int ow = (int)(v % g.Wo); v /= g.Wo;
    int oh = (int)(v % g.Ho); v /= g.Ho;
    int od = (int)(v % g.Do);
    int n = (int)(v / g.Do);
    float acc = 0.f;
    for (int kd = 0; kd < g.kD; ++kd) {
        int id = od * g.sD - g.pD + kd;
        if (id < 0 || id >= g.D) continue;
        for (int kh = 0; kh < g.kH; ++kh) {
            int ih = oh * g.sH - g.pH + kh;
            if (ih < 0 || ih >= g.H) continue;
            for (int kw = 0; kw < g.kW; ++kw) {
                int iw = ow * g.sW - g.pW + kw;
                if (iw < 0 || iw >= g.W) continue;
                const T* xp = x + ((((long long)n * g.D + id) * g.H + ih) * g.W + iw) * g.Cin;
                const T* wp = w + ((((long long)co * g.kD + kd) * g.kH + kh) * g.kW + kw) * g.Cin;
                for (int ci = 0; ci < g.Cin; ++ci) acc = fmaf(Elem<T>::load(xp + ci), Elem<T>::load(wp + ci), acc);
            }
        }
    }
    Elem<T>::store(y + idx, acc);
}

template <typename T>
__global__ void __launch_bounds__(256) dgrad_kernel(Geom g, const T* __restrict__ dy, const T* __restrict__ w, T* __restrict__ dx) {
    long long total = g.in_voxels() * g.Cin;
    long long idx = (long long)blockIdx.x * 256 + threadIdx.x;
    if (idx >= total) return;
    int ci = (int)(idx % g.Cin);
    long long v = idx / g.Cin;
    int iw = (int)(v % g.W); v /= g.W;
    int ih = (int)(v % g.H); v /= g.H;
    int id = (int)(v % g.D);
    int n = (int)(v / g.D);
    float acc = 0.f;
    for (int kd = 0; kd < g.kD; ++kd) {
        int nd = id + g.pD - kd;
        if (nd < 0 || nd % g.sD) continue;
        int od = nd / g.sD;
        if (od >= g.Do) continue;
        for (int kh = 0; kh < g.kH; ++kh) {
            int nh = ih + g.pH - kh;
            if (nh < 0 || nh % g.sH) continue;
            int oh = nh / g.sH;
            if (oh >= g.Ho) continue;
            for (int kw = 0; kw < g.kW; ++kw) {
                int nw = iw + g.pW - kw;
                if (nw < 0 || nw % g.sW) continue;
                int ow = nw / g.sW;
                if (ow >= g.Wo) continue;
                const T* gp = dy + ((((long long)n * g.Do + od) * g.Ho + oh) * g.Wo + ow) * g.Cout;
                const T* wp = w + (((long long)kd * g.kH + kh) * g.kW + kw) * g.Cin + ci;
                long long wstride = g.taps() * g.Cin;
                for (int co = 0; co < g.Cout; ++co) acc = fmaf(Elem<T>::load(gp + co), Elem<T>::load(wp + co * wstride), acc);
            }
        }
    }
    Elem<T>::store(dx + idx, acc);
}

// Stage 1 of wgrad: block (pair-block, tap, chunk); each thread owns one
// (co, ci) pair and sums over the output voxels of its chunk.
template <typename T>
__global__ void __launch_bounds__(256) wgrad_partial_kernel(Geom g, const T* __restrict__ x, const T* __restrict__ dy,
                                                            float* __restrict__ part, long long chunk_len) {
    int pair = blockIdx.x * 256 + threadIdx.x;
    int t = blockIdx.y;
    int chunk = blockIdx.z;
    if (pair >= g.Cout * g.Cin) return;
    int co = pair / g.Cin, ci = pair % g.Cin;
    int kd = t / (g.kH * g.kW), kh = (t / g.kW) % g.kH, kw = t % g.kW;
    long long v0 = (long long)chunk * chunk_len;
    long long v1 = v0 + chunk_len;
    long long P = g.out_voxels();
    if (v1 > P) v1 = P;
    float acc = 0.f;
    for (long long v = v0; v < v1; ++v) {
        long long r = v;
        int ow = (int)(r % g.Wo); r /= g.Wo;
        int oh = (int)(r % g.Ho); r /= g.Ho;
        int od = (int)(r % g.Do);
        int n = (int)(r / g.Do);
        int id = od * g.sD - g.pD + kd, ih = oh * g.sH - g.pH + kh, iw = ow * g.sW - g.pW + kw;
        if (id < 0 || id >= g.D || ih < 0 || ih >= g.H || iw < 0 || iw >= g.W) continue;
        float a = Elem<T>::load(dy + v * g.Cout + co);
        float b = Elem<T>::load(x + ((((long long)n * g.D + id) * g.H + ih) * g.W + iw) * g.Cin + ci);
        acc = fmaf(a, b, acc);
    }
    part[(long long)chunk * g.w_elems() + ((long long)co * g.taps() + t) * g.Cin + ci] = acc;
}

}  // namespace

// Sums `parts` partial tensors of `n` floats each in a fixed order
// (bit-reproducible): a block handles 16 elements; thread (g, e) adds parts
// g, g + 16, g + 32, ... of element e, then the 16 group sums are added in
// index order.  Shared by every split-K weight-gradient kernel.
__global__ void __launch_bounds__(256) reduce_partials_kernel(const float* __restrict__ part, float* __restrict__ out,
                                                              long long n, int parts) {
    __shared__ float sm[16][17];
    const int e = threadIdx.x & 15, g = threadIdx.x >> 4;
    const long long i = (long long)blockIdx.x * 16 + e;
    float acc = 0.f;
    if (i < n)
        for (int p = g; p < parts; p += 16) acc += part[(long long)p * n + i];
    sm[g][e] = acc;
    __syncthreads();
    if (g == 0 && i < n) {
        float a = 0.f;
#pragma unroll
        for (int k = 0; k < 16; ++k) a += sm[k][e];
        out[i] = a;
    }
}

// The same sums in the same order, four consecutive elements per thread: a block handles 64 elements and each of its
// loads covers 256 contiguous bytes per group instead of 64.
__global__ void __launch_bounds__(256) reduce_partials4_kernel(const float* __restrict__ part, float* __restrict__ out,
                                                               long long n4, long long n, int parts) {
    __shared__ float4 sm[16][17];
    const int e = threadIdx.x & 15, g = threadIdx.x >> 4;
    const long long i = (long long)blockIdx.x * 16 + e;
    float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
    if (i < n4)
        for (int p = g; p < parts; p += 16) {
            const float4 b = *(const float4*)(part + (long long)p * n + 4 * i);
            acc.x += b.x; acc.y += b.y; acc.z += b.z; acc.w += b.w;
        }
    sm[g][e] = acc;
    __syncthreads();
    if (g == 0 && i < n4) {
        float4 a = make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
        for (int k = 0; k < 16; ++k) {
            const float4 b = sm[k][e];
            a.x += b.x; a.y += b.y; a.z += b.z; a.w += b.w;
        }
        *(float4*)(out + 4 * i) = a;
    }
}

// Few partial tensors of many elements (the deep layers: two to sixteen slots of millions of weights): one thread
// per four consecutive elements adds the parts in index order.  The 16-groups kernel above would launch a block per
// 16 elements with most of its threads idle (71 us for 2 x 3.5 M floats against 12 us here).
__global__ void __launch_bounds__(256) reduce_few_partials_kernel(const float* __restrict__ part, float* __restrict__ out, long long n4, long long n,
                                                                  int parts) {
    const long long i = (long long)blockIdx.x * 256 + threadIdx.x;
    if (i >= n4) return;
    float4 a = *(const float4*)(part + 4 * i);
    for (int p = 1; p < parts; ++p) {
        const float4 b = *(const float4*)(part + (long long)p * n + 4 * i);
        a.x += b.x; a.y += b.y; a.z += b.z; a.w += b.w;
    }
    *(float4*)(out + 4 * i) = a;
}

// out[i] = sum over parts of part[p * n + i], in an order that depends only on (n, parts)
int reduce_partials(const float* part, float* out, long long n, int parts, hipStream_t s) {
    if (parts <= 16 && n % 4 == 0 && n >= (1 << 16) && (((uintptr_t)part | (uintptr_t)out) & 15) == 0)
        reduce_few_partials_kernel<<<(unsigned)((n / 4 + 255) / 256), 256, 0, s>>>(part, out, n / 4, n, parts);
    else if (n % 4 == 0 && n >= 4096 && (((uintptr_t)part | (uintptr_t)out) & 15) == 0)
        reduce_partials4_kernel<<<(unsigned)((n / 4 + 15) / 16), 256, 0, s>>>(part, out, n / 4, n, parts);
    else
        reduce_partials_kernel<<<(unsigned)((n + 15) / 16), 256, 0, s>>>(part, out, n, parts);
    return check_launch();
}

static void wgrad_chunks(const Geom& g, int* chunks, long long* chunk_len) {
    long long P = g.out_voxels();
    long long c = (P + 2047) / 2048;
    if (c > 256) c = 256;
    long long cap = (128ll << 20) / (g.w_elems() * 4);
    if (cap < 1) cap = 1;
    if (c > cap) c = cap;
    if (c < 1) c = 1;
    *chunk_len = (P + c - 1) / c;
    *chunks = (int)((P + *chunk_len - 1) / *chunk_len);
}

size_t direct_workspace_bytes(const Geom& g, int pass) {
    if (pass != MI3D_PASS_WGRAD) return 0;
    int chunks; long long len;
    wgrad_chunks(g, &chunks, &len);
    return (size_t)chunks * g.w_elems() * sizeof(float);
}

static bool grid_ok(long long total) { return (total + 255) / 256 <= 0x7fffffffll; }

int direct_fwd(const Geom& g, const void* x, const void* w, void* y, hipStream_t s) {
    long long total = g.out_voxels() * g.Cout;
    if (!grid_ok(total)) return MI3D_ERR_UNSUPPORTED;
    unsigned blocks = (unsigned)((total + 255) / 256);
    if (g.dtype == MI3D_F32) fwd_kernel<float><<<blocks, 256, 0, s>>>(g, (const float*)x, (const float*)w, (float*)y);
    else fwd_kernel<uint16_t><<<blocks, 256, 0, s>>>(g, (const uint16_t*)x, (const uint16_t*)w, (uint16_t*)y);
    return check_launch();
}

int direct_dgrad(const Geom& g, const void* dy, const void* w, void* dx, hipStream_t s) {
    long long total = g.in_voxels() * g.Cin;
    if (!grid_ok(total)) return MI3D_ERR_UNSUPPORTED;
    unsigned blocks = (unsigned)((total + 255) / 256);
    if (g.dtype == MI3D_F32) dgrad_kernel<float><<<blocks, 256, 0, s>>>(g, (const float*)dy, (const float*)w, (float*)dx);
    else dgrad_kernel<uint16_t><<<blocks, 256, 0, s>>>(g, (const uint16_t*)dy, (const uint16_t*)w, (uint16_t*)dx);
    return check_launch();
}

int direct_wgrad(const Geom& g, const void* x, const void* dy, float* dw, void* ws, size_t ws_bytes, hipStream_t s) {
    int chunks; long long len;
    wgrad_chunks(g, &chunks, &len);
    if (ws_bytes < (size_t)chunks * g.w_elems() * sizeof(float)) return MI3D_ERR_WORKSPACE;
    long long pairs = (long long)g.Cout * g.Cin;
    if (g.taps() > 65535 || chunks > 65535) return MI3D_ERR_UNSUPPORTED;
    dim3 grid((unsigned)((pairs + 255) / 256), (unsigned)g.taps(), (unsigned)chunks);
    float* part = (float*)ws;
    if (g.dtype == MI3D_F32) wgrad_partial_kernel<float><<<grid, 256, 0, s>>>(g, (const float*)x, (const float*)dy, part, len);
    else wgrad_partial_kernel<uint16_t><<<grid, 256, 0, s>>>(g, (const uint16_t*)x, (const uint16_t*)dy, part, len);
    int st = check_launch();
    if (st) return st;
    long long n = g.w_elems();
    return reduce_partials(part, dw, n, chunks, s);
}

}  // namespace mi3d
