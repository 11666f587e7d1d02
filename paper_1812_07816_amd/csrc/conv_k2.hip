// 2x2x2 / stride 2 / pad 0 convolution (the decoder's up-sampling layers of
// the network of Section 4.1, run with roles swapped): forward and data
// gradient on bf16 MFMA (v_mfma_f32_32x32x16_bf16), fp32 accumulation.
//
// The taps do not overlap, so both passes are plain matrix products with a
// gather or a scatter on the big-volume side:
//   forward  y[o, co]      = sum_{t, ci} x[2 o + t, ci] w[co, t, ci]     K = 8 Cin, gathered from 8 voxels
//   dgrad    dx[2 o + t, ci] = sum_co dy[o, co] w[co, t, ci]             K = Cout, scattered to 8 voxels
// A (MFMA rows) = a panel of weights: G blocks of 32 output channels x all of
// K, packed as fragments and kept in LDS by a workgroup for its whole life;
// B (MFMA columns) = 32 voxels of the small volume per wave, whose fragments
// (8 consecutive channels = 16 bytes in NDHWC) are loaded straight from global
// memory into registers through a ring four k-steps deep.  A lane ends with
// consecutive output channels of one voxel (two 16-byte stores after a
// v_permlane32_swap), at the voxel's own address (forward) or at the address of
// voxel 2 o + t (data gradient).  Workgroups are persistent: workgroup g owns
// the panel g % NG and walks tiles of 128 small-volume voxels.
#include "mi3d_internal.h"

namespace mi3d {
namespace {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;
typedef __attribute__((__vector_size__(2 * sizeof(float)))) float f32x2;
typedef __attribute__((__vector_size__(2 * sizeof(__bf16)))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(2))) unsigned u32x2;

struct K2Params {
    const uint16_t* in;     // forward: x (big volume, Cb channels); dgrad: dy (small volume, Cs channels)
    const uint16_t* wpack;  // [block of 32 output channels][k16 step][lane][8]
    uint16_t* out;          // forward: y (small volume); dgrad: dx (big volume)
    uint16_t* dump;         // 2 KB that masked store lanes write to
    int N, Ds, Hs, Ws;      // small volume
    int Cs, Cb;             // channels of the small-volume / big-volume tensor (Cout / Cin of the convolution)
    int K16;                // k-steps of 16
    int NG;                 // panels (groups of G blocks)
    long long vox;          // N * Ds * Hs * Ws
    int nwg;
};

// MODE 0: forward (gather), MODE 1: data gradient (scatter).  G: blocks of 32 output channels per panel.
template <int MODE, int G>
__global__ void __launch_bounds__(256, MODE == 1 ? 2 : 1) k2_kernel(K2Params P) {
    extern __shared__ __attribute__((aligned(16))) char panel[];   // G * K16 KB
    const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
    const int group = blockIdx.x % P.NG, first_tile = blockIdx.x / P.NG, tile_step = P.nwg / P.NG;
    {
        const uint4* src = (const uint4*)P.wpack + (long long)group * G * P.K16 * 64;
        for (int i = t; i < G * P.K16 * 64; i += 256) ((uint4*)panel)[i] = src[i];
    }
    __syncthreads();
    const char* a_lane = panel + lane * 16;
    const long long tiles = (P.vox + 127) / 128;
    const int h = lane >> 5;
    const int cb16 = P.Cb / 16;   // k-steps per tap (forward)

    for (long long tile = first_tile; tile < tiles; tile += tile_step) {
        const long long v = tile * 128 + wave * 32 + (lane & 31);
        const bool ok = v < P.vox;
        long long r = ok ? v : 0;
        const int ow = (int)(r % P.Ws); r /= P.Ws;
        const int oh = (int)(r % P.Hs); r /= P.Hs;
        const int od = (int)(r % P.Ds);
        const int n = (int)(r / P.Ds);
        // element offset of big-volume voxel 2 o (tap 0); tap (td, th, tw) adds ((td * Hb + th) * Wb + tw) * Cb
        const long long Hb = 2ll * P.Hs, Wb = 2ll * P.Ws;
        const long long big0 = ((((long long)n * 2 * P.Ds + 2 * od) * Hb + 2 * oh) * Wb + 2 * ow) * P.Cb;
        auto tap_off = [&](int tap) { return (((long long)(tap >> 2) * Hb + ((tap >> 1) & 1)) * Wb + (tap & 1)) * P.Cb; };
        const uint16_t* src = MODE == 0 ? P.in + big0 + 8 * h : P.in + (ok ? v : 0) * P.Cs + 8 * h;
        auto load_b = [&](int kk) -> uint4 {
            if (MODE == 0) {
                const int tap = kk / cb16, c = (kk - tap * cb16) * 16;
                return *(const uint4*)(src + tap_off(tap) + c);
            }
            return *(const uint4*)(src + kk * 16);
        };
        f32x16 acc[G];
#pragma unroll
        for (int g = 0; g < G; ++g)
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[g][i] = 0.f;
        uint4 ring[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) ring[i] = load_b(i);
        for (int kk0 = 0; kk0 < P.K16; kk0 += 4) {
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const bf16x8 b = __builtin_bit_cast(bf16x8, ring[i]);
                const int nxt = kk0 + 4 + i;
                ring[i] = load_b(nxt < P.K16 ? nxt : P.K16 - 1);   // unconditional (the last ones are re-reads nobody uses)
#pragma unroll
                for (int g = 0; g < G; ++g) {
                    const bf16x8 a = *(const bf16x8*)(a_lane + ((long long)(g * P.K16 + kk0 + i)) * 1024);
                    acc[g] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[g], 0, 0, 0);
                }
            }
        }
        // stores: lane (voxel, half h) ends with channels 16 h .. 16 h + 15 of each block
#pragma unroll
        for (int g = 0; g < G; ++g) {
            uint32_t o[8];
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                f32x2 p2 = {acc[g][2 * i], acc[g][2 * i + 1]};
                o[i] = __builtin_bit_cast(uint32_t, __builtin_convertvector(p2, bf16x2));
            }
            uint4 c[2];
#pragma unroll
            for (int k = 0; k < 2; ++k) {
                u32x2 s0 = __builtin_amdgcn_permlane32_swap(o[2 * k], o[2 * k + 4], false, false);
                u32x2 s1 = __builtin_amdgcn_permlane32_swap(o[2 * k + 1], o[2 * k + 5], false, false);
                c[k].x = s0[0]; c[k].y = s1[0]; c[k].z = s0[1]; c[k].w = s1[1];
            }
            const int nb = group * G + g;     // block of 32 output channels
            uint16_t* dst;
            if (MODE == 0) {
                dst = P.out + v * P.Cs + nb * 32 + 16 * h;
            } else {
                const int per_tap = P.Cb / 32;
                const int tap = nb / per_tap, c0 = (nb - tap * per_tap) * 32;
                dst = P.out + big0 + tap_off(tap) + c0 + 16 * h;
            }
            uint16_t* q = ok ? dst : P.dump + lane * 16;
            *(uint4*)q = c[0];
            *(uint4*)(q + 8) = c[1];
        }
    }
}

// [Cout][2][2][2][Cin] -> A fragments.  MODE 0: block = 32 couts, k = tap * Cin + ci.  MODE 1: block nb = (tap, 32 cins), k = cout.
__global__ void __launch_bounds__(256) k2_pack_kernel(const uint16_t* __restrict__ w, uint16_t* __restrict__ wpack, int Cin, int Cout, int mode) {
    const long long total = 8ll * Cin * Cout;
    const long long idx = (long long)blockIdx.x * 256 + threadIdx.x;
    if (idx >= total) return;
    const int j = (int)(idx & 7);
    long long r = idx >> 3;
    const int lane = (int)(r & 63); r >>= 6;
    const int K16 = mode == 0 ? Cin / 2 : Cout / 16;
    const int kk = (int)(r % K16);
    const int nb = (int)(r / K16);
    const int m = lane & 31, k = 16 * kk + 8 * (lane >> 5) + j;
    int co, tap, ci;
    if (mode == 0) {
        co = nb * 32 + m; tap = k / Cin; ci = k - tap * Cin;
    } else {
        const int per_tap = Cin / 32;
        tap = nb / per_tap; ci = (nb - tap * per_tap) * 32 + m; co = k;
    }
    wpack[idx] = w[((long long)co * 8 + tap) * Cin + ci];
}

int pick_g(int blocks, int K16, int max_kb) {   // largest G in {4, 2, 1} that divides the block count and fits the panel
    for (int g = 4; g >= 1; g >>= 1)
        if (blocks % g == 0 && g * K16 <= max_kb) return g;
    return 0;
}

}  // namespace

bool k2_supported(const Geom& g, int pass) {
    if (pass == MI3D_PASS_WGRAD) return false;
    if (g.dtype != MI3D_BF16 || g.kD != 2 || g.kH != 2 || g.kW != 2) return false;
    if (g.sD != 2 || g.sH != 2 || g.sW != 2 || g.pD || g.pH || g.pW) return false;
    if ((g.D | g.H | g.W) & 1) return false;
    if (g.Cin % 32 || g.Cout % 64) return false;   // k-steps come in fours (the register ring)
    if (pass == MI3D_PASS_FWD) return pick_g(g.Cout / 32, g.Cin / 2, 128) > 0;
    return pick_g(g.Cin / 4, g.Cout / 16, 64) > 0;
}

size_t k2_workspace_bytes(const Geom& g, int pass) {
    return k2_supported(g, pass) ? (((size_t)g.w_elems() * 2 + 255) & ~(size_t)255) + 2048 : 0;
}

int k2_conv(const Geom& g, int pass, const void* a, const void* w, void* out, void* ws, size_t ws_bytes, hipStream_t s) {
    if (!k2_supported(g, pass)) return MI3D_ERR_UNSUPPORTED;
    if (ws_bytes < k2_workspace_bytes(g, pass)) return MI3D_ERR_WORKSPACE;
    const int mode = pass == MI3D_PASS_FWD ? 0 : 1;
    const long long total = g.w_elems();
    k2_pack_kernel<<<(unsigned)((total + 255) / 256), 256, 0, s>>>((const uint16_t*)w, (uint16_t*)ws, g.Cin, g.Cout, mode);
    int st = check_launch();
    if (st) return st;
    K2Params P;
    P.in = (const uint16_t*)a; P.wpack = (const uint16_t*)ws; P.out = (uint16_t*)out;
    P.dump = (uint16_t*)((char*)ws + (((size_t)g.w_elems() * 2 + 255) & ~(size_t)255));
    P.N = g.N; P.Ds = g.Do; P.Hs = g.Ho; P.Ws = g.Wo; P.Cs = g.Cout; P.Cb = g.Cin;
    P.vox = (long long)g.N * g.Do * g.Ho * g.Wo;
    int blocks, G;
    if (mode == 0) { P.K16 = g.Cin / 2; blocks = g.Cout / 32; G = pick_g(blocks, P.K16, 128); }
    else { P.K16 = g.Cout / 16; blocks = g.Cin / 4; G = pick_g(blocks, P.K16, 64); }
    P.NG = blocks / G;
    const long long tiles = (P.vox + 127) / 128;
    int dev = 0, cus = 256;
    if (hipGetDevice(&dev) == hipSuccess) (void)hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev);
    // a multiple of NG workgroups, about one (forward) or two (data gradient) per CU, no more than there are units
    long long per_group = (long long)(mode == 0 ? cus : 2 * cus) / P.NG;
    if (per_group < 1) per_group = 1;
    if (per_group > tiles) per_group = tiles;
    P.nwg = (int)(per_group * P.NG);
    const size_t lds = (size_t)G * P.K16 * 1024;
    static bool attr_set = false;
    if (!attr_set) {
        hipError_t e = hipSuccess;
        const void* fns0[3] = {(const void*)k2_kernel<0, 1>, (const void*)k2_kernel<0, 2>, (const void*)k2_kernel<0, 4>};
        const void* fns1[3] = {(const void*)k2_kernel<1, 1>, (const void*)k2_kernel<1, 2>, (const void*)k2_kernel<1, 4>};
        for (int i = 0; i < 3 && e == hipSuccess; ++i) e = hipFuncSetAttribute(fns0[i], hipFuncAttributeMaxDynamicSharedMemorySize, 128 * 1024);
        for (int i = 0; i < 3 && e == hipSuccess; ++i) e = hipFuncSetAttribute(fns1[i], hipFuncAttributeMaxDynamicSharedMemorySize, 64 * 1024);
        if (e != hipSuccess) { note_hip_error(e); return MI3D_ERR_HIP; }
        attr_set = true;
    }
#define K2_LAUNCH(M, GG) k2_kernel<M, GG><<<(unsigned)P.nwg, 256, lds, s>>>(P)
    if (mode == 0) { if (G == 4) K2_LAUNCH(0, 4); else if (G == 2) K2_LAUNCH(0, 2); else K2_LAUNCH(0, 1); }
    else { if (G == 4) K2_LAUNCH(1, 4); else if (G == 2) K2_LAUNCH(1, 2); else K2_LAUNCH(1, 1); }
#undef K2_LAUNCH
    return check_launch();
}

}  // namespace mi3d
