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
//
// The big-volume tensor (x of the forward pass and of the weight gradient, dx of the data gradient) may be a
// channel range of a wider tensor: `pitch` channels per voxel, the operand starting at channel `offset`.  The
// decoder uses that to up-sample straight into the concatenated tensor and to read the up-sampled half of its
// gradient in place.
//
// Weight gradient: dw[co][t][ci] = sum_o dy[o][co] x[2 o + t][ci], a contraction over the small-volume voxels with
// both operands transposed on the way (ds_read_b64_tr_b16 from [16-channel slab][voxel] tiles in LDS, as in the
// 3x3x3 weight-gradient kernels).  A workgroup owns 64 couts x 32 cins x 8 taps (wave w: taps 2w, 2w + 1) and a
// range of voxels, staged 64 at a time (double buffered); partial sums per workgroup, added in a fixed order.
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
    int pb, ob;             // big-volume tensor: channels per voxel in memory, first channel of the operand
    int K16;                // k-steps of 16
    int NG;                 // panels (groups of G blocks)
    long long vox;          // N * Ds * Hs * Ws
    int nwg;
};

// MODE 0: forward (gather), MODE 1: data gradient (scatter).  G: blocks of 32 output channels per panel.
// ROWS (MODE 1, G = 4, 32 big-volume channels: a panel is the four taps (kh, kw) of one kd): the scattered voxels of a
// wave's 32 small voxels are two runs of 64 neighbouring big voxels (rows 2 oh and 2 oh + 1); the wave passes them
// through LDS so that a store instruction writes whole 64-byte voxels of 16 neighbours (four lanes per voxel) instead
// of 16-byte pieces of 64 voxels.
constexpr int K2_STG = 8192 + 256;   // per wave: 2 rows x 64 voxels x 64 B, and the 32 voxels' offsets
template <int MODE, int G, bool ROWS = false>
__global__ void __launch_bounds__(256, MODE == 1 ? 2 : 1) k2_kernel(K2Params P) {
    extern __shared__ __attribute__((aligned(16))) char panel[];   // G * K16 KB (+ 4 x K2_STG with ROWS)
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

    // Per-tile addressing of this lane's voxel: v (small volume), element offset of big-volume voxel 2 o (tap 0).
    const long long Hb = 2ll * P.Hs, Wb = 2ll * P.Ws;
    auto tap_off = [&](int tap) { return (((long long)(tap >> 2) * Hb + ((tap >> 1) & 1)) * Wb + (tap & 1)) * P.pb; };
    struct Where { long long v, big0; bool ok; };
    auto locate = [&](long long tile) {
        Where w;
        w.v = tile * 128 + wave * 32 + (lane & 31);
        w.ok = tile < tiles && w.v < P.vox;
        int r = w.ok ? (int)w.v : 0;             // the small volume has fewer than 2^31 voxels
        const int ow = r % P.Ws; r /= P.Ws;
        const int oh = r % P.Hs; r /= P.Hs;
        const int od = r % P.Ds;
        const int n = r / P.Ds;
        w.big0 = ((((long long)n * 2 * P.Ds + 2 * od) * Hb + 2 * oh) * Wb + 2 * ow) * P.pb + P.ob;
        return w;
    };
    auto source = [&](const Where& w) { return MODE == 0 ? P.in + w.big0 + 8 * h : P.in + (w.ok ? w.v : 0) * P.Cs + 8 * h; };
    auto load_b = [&](const uint16_t* src, int kk) -> uint4 {
        if (MODE == 0) {
            const int tap = kk / cb16, c = (kk - tap * cb16) * 16;
            return *(const uint4*)(src + tap_off(tap) + c);
        }
        return *(const uint4*)(src + kk * 16);
    };

    // The B fragments run through a ring four k-steps deep that does not stop at tile ends: the last four steps of a
    // tile fetch the first four of the workgroup's next tile, so a tile starts with its operands in registers
    // (without this every tile began with an exposed load latency).
    Where cur = locate(first_tile);
    const uint16_t* src = source(cur);
    uint4 ring[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) ring[i] = load_b(src, i);
    for (long long tile = first_tile; tile < tiles; tile += tile_step) {
        const Where nxt_w = locate(tile + tile_step);      // past the end: voxel 0, loaded and never used
        const uint16_t* src_next = source(nxt_w);
        f32x16 acc[G];
#pragma unroll
        for (int g = 0; g < G; ++g)
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[g][i] = 0.f;
        for (int kk0 = 0; kk0 < P.K16; kk0 += 4) {
            const bool last = kk0 + 4 >= P.K16;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const bf16x8 b = __builtin_bit_cast(bf16x8, ring[i]);
                ring[i] = load_b(last ? src_next : src, last ? i : kk0 + 4 + i);   // unconditional
#pragma unroll
                for (int g = 0; g < G; ++g) {
                    const bf16x8 a = *(const bf16x8*)(a_lane + ((long long)(g * P.K16 + kk0 + i)) * 1024);
                    acc[g] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[g], 0, 0, 0);
                }
            }
        }
        // stores: lane (voxel, half h) ends with channels 16 h .. 16 h + 15 of each block
        char* stg = panel + (size_t)G * P.K16 * 1024 + (ROWS ? wave * K2_STG : 0);
        if constexpr (ROWS) {
            if (lane < 32) ((long long*)(stg + 8192))[lane] = cur.ok ? cur.big0 : -1;
        }
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
            if constexpr (ROWS) {   // block g is tap (kh, kw) = (g / 2, g % 2): big voxel 2 v + kw of row kh of the wave's run
                char* q = stg + (g >> 1) * 4096 + (2 * (lane & 31) + (g & 1)) * 64 + h * 32;
                *(uint4*)q = c[0];
                *(uint4*)(q + 16) = c[1];
                continue;
            }
            const int nb = group * G + g;     // block of 32 output channels
            uint16_t* dst;
            if (MODE == 0) {
                dst = P.out + cur.v * P.Cs + nb * 32 + 16 * h;
            } else {
                const int per_tap = P.Cb / 32;
                const int tap = nb / per_tap, c0 = (nb - tap * per_tap) * 32;
                dst = P.out + cur.big0 + tap_off(tap) + c0 + 16 * h;
            }
            uint16_t* q = cur.ok ? dst : P.dump + lane * 16;
            *(uint4*)q = c[0];
            *(uint4*)(q + 8) = c[1];
        }
        if constexpr (ROWS) {
            // same wave, LDS executes in order: only the compiler must not move the reads above the writes
            asm volatile("" ::: "memory");
            __builtin_amdgcn_wave_barrier();
            asm volatile("" ::: "memory");
#pragma unroll
            for (int kh = 0; kh < 2; ++kh)
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const uint4 v = *(const uint4*)(stg + kh * 4096 + i * 1024 + lane * 16);
                    const int bv = i * 16 + (lane >> 2);                       // big voxel of the run; its small voxel is bv / 2
                    const long long b0 = ((const long long*)(stg + 8192))[bv >> 1];
                    uint16_t* dst = P.out + b0 + tap_off(group * 4 + kh * 2 + (bv & 1)) + (lane & 3) * 8;
                    *(uint4*)(b0 >= 0 ? dst : P.dump + lane * 8) = v;
                }
            asm volatile("" ::: "memory");
            __builtin_amdgcn_wave_barrier();   // the next tile's writes stay behind these reads
            asm volatile("" ::: "memory");
        }
        cur = nxt_w;
        src = src_next;
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


// ---- weight gradient --------------------------------------------------------------------------------------
typedef __attribute__((__vector_size__(4 * sizeof(short)))) short s16x4;
typedef __attribute__((__vector_size__(8 * sizeof(short)))) short s16x8;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float f32x4;

constexpr int WV = 64;                              // small-volume voxels per stage
constexpr int WCO = 64, WCI = 32;                   // channel block of a workgroup
constexpr int DY_STAGE = (WCO / 16) * WV * 32;      // 4 slabs x 64 voxels x 32 bytes
constexpr int X_STAGE = 8 * (WCI / 16) * WV * 32;   // 8 taps x 2 slabs x 64 voxels x 32 bytes
constexpr int W_STAGE = DY_STAGE + X_STAGE;         // 40 KB

struct K2WgParams {
    const uint16_t* x;      // big volume (a channel range of a tensor with xpitch channels per voxel)
    const uint16_t* dy;     // small volume, Cs channels
    float* part;            // [slot][Cs][8][Cb]
    int Ds, Hs, Ws, Cs, Cb, xpitch, xoff;
    int vox;                // N * Ds * Hs * Ws
    int CiT;                // cin blocks
    int slots;              // workgroups per (cout block, cin block) pair
};

// 16 channels x 32 voxels from a [voxel][16 channels] slab: lane group g = lane / 16 gets voxels 4g .. 4g + 3 and
// 16 + 4g .. 16 + 4g + 3 of channel lane % 16 (the same permutation of the contraction index for both operands)
__device__ __forceinline__ bf16x8 tr_frag(const char* p) {
    typedef __attribute__((address_space(3))) s16x4* lptr;
    s16x4 a = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lptr)(p));
    s16x4 b = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lptr)(p + 16 * 32));
    s16x8 c = __builtin_shufflevector(a, b, 0, 1, 2, 3, 4, 5, 6, 7);
    return __builtin_bit_cast(bf16x8, c);
}

__global__ void __launch_bounds__(256, 2) k2_wgrad_kernel(K2WgParams P) {
    extern __shared__ __attribute__((aligned(16))) char lds[];   // two stages
    const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
    const int pair = blockIdx.y, slot = blockIdx.x;
    const int cot = pair / P.CiT, cit = pair % P.CiT;
    const int stages = (P.vox + WV - 1) / WV;
    const int s0 = (int)((long long)stages * slot / P.slots), s1 = (int)((long long)stages * (slot + 1) / P.slots);

    // staging plan.  x: piece c = t % 4 (8 channels) of voxel j = t / 4, once per tap; dy: piece c8 = t % 8 of voxels
    // t / 8 and t / 8 + 32.  Loads are unconditional (voxels past the end read voxel 0 and are zeroed on the way to LDS).
    const int c = t & 3, j = t >> 2, c8 = t & 7, j2 = t >> 3;
    const long long Hb = 2ll * P.Hs, Wb = 2ll * P.Ws;
    typedef __attribute__((ext_vector_type(4))) unsigned u32x4;
    u32x4 px[8], pdy[2];
    unsigned okbits = 0;
    auto load_stage = [&](int s) {
        const int v = s * WV + j;
        const bool ok = v < P.vox;
        int r = ok ? v : 0;
        const int ow = r % P.Ws; r /= P.Ws;
        const int oh = r % P.Hs; r /= P.Hs;
        const int od = r % P.Ds;
        const int n = r / P.Ds;
        const uint16_t* src = P.x + ((((long long)n * 2 * P.Ds + 2 * od) * Hb + 2 * oh) * Wb + 2 * ow) * P.xpitch + P.xoff + cit * WCI + c * 8;
#pragma unroll
        for (int tap = 0; tap < 8; ++tap)
            px[tap] = *(const u32x4*)(src + (((long long)(tap >> 2) * Hb + ((tap >> 1) & 1)) * Wb + (tap & 1)) * P.xpitch);
        okbits = ok ? 1u : 0u;
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            const int v2 = s * WV + j2 + 32 * i;
            const bool ok2 = v2 < P.vox;
            pdy[i] = *(const u32x4*)(P.dy + (long long)(ok2 ? v2 : 0) * P.Cs + cot * WCO + c8 * 8);
            okbits |= (ok2 ? 2u : 0u) << i;
        }
    };
    auto write_stage = [&](int buf) {
        char* dyb = lds + buf * W_STAGE;
        char* xb = dyb + DY_STAGE;
        const unsigned mx = (okbits & 1u) ? ~0u : 0u;
#pragma unroll
        for (int tap = 0; tap < 8; ++tap)
            *(u32x4*)(xb + ((tap * 2 + (c >> 1)) * WV + j) * 32 + (c & 1) * 16) = px[tap] & mx;
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            const unsigned md = ((okbits >> (1 + i)) & 1u) ? ~0u : 0u;
            *(u32x4*)(dyb + ((c8 >> 1) * WV + j2 + 32 * i) * 32 + (c8 & 1) * 16) = pdy[i] & md;
        }
    };

    f32x4 acc[2][4][2];   // [tap of the wave][cout slab][cin slab]
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int b = 0; b < 4; ++b)
#pragma unroll
            for (int d = 0; d < 2; ++d) acc[a][b][d] = f32x4{0.f, 0.f, 0.f, 0.f};
    const int g = lane >> 4, sl = lane & 15;
    const int lane_off = (4 * g + (sl >> 2)) * 32 + (sl & 3) * 8;

    if (s0 < s1) {
        load_stage(s0);
        write_stage(0);
    }
    __syncthreads();
    for (int s = s0; s < s1; ++s) {
        const int buf = (s - s0) & 1;
        load_stage(s + 1 < s1 ? s + 1 : s);   // unconditional; after the last stage: fetched, never used
        __builtin_amdgcn_sched_barrier(0);
        const char* dyb = lds + buf * W_STAGE + lane_off;
        const char* xb = dyb + DY_STAGE;
#pragma unroll
        for (int kc = 0; kc < WV / 32; ++kc) {
            bf16x8 a[4];
#pragma unroll
            for (int q = 0; q < 4; ++q) a[q] = tr_frag(dyb + (q * WV + kc * 32) * 32);
#pragma unroll
            for (int tt = 0; tt < 2; ++tt)
#pragma unroll
                for (int cs = 0; cs < 2; ++cs) {
                    const bf16x8 b = tr_frag(xb + (((2 * wave + tt) * 2 + cs) * WV + kc * 32) * 32);
#pragma unroll
                    for (int q = 0; q < 4; ++q) acc[tt][q][cs] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[q], b, acc[tt][q][cs], 0, 0, 0);
                }
        }
        __builtin_amdgcn_sched_barrier(0);
        write_stage(buf ^ 1);   // its readers passed the barrier of the previous stage
        __syncthreads();
    }
    // C layout of the 16x16 tile: column lane % 16 = cin, row 4 (lane / 16) + v = cout
    float* out = P.part + (long long)slot * P.Cs * 8 * P.Cb;
#pragma unroll
    for (int tt = 0; tt < 2; ++tt)
#pragma unroll
        for (int q = 0; q < 4; ++q)
#pragma unroll
            for (int cs = 0; cs < 2; ++cs)
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    const int co = cot * WCO + q * 16 + 4 * (lane >> 4) + v;
                    const int ci = cit * WCI + cs * 16 + (lane & 15);
                    out[((long long)co * 8 + 2 * wave + tt) * P.Cb + ci] = acc[tt][q][cs][v];
                }
}

static int k2_wgrad_slots(const Geom& g) {
    const int pairs = (g.Cout / WCO) * (g.Cin / WCI);
    const long long vox = (long long)g.N * g.Do * g.Ho * g.Wo;
    const long long stages = (vox + WV - 1) / WV;
    int dev = 0, cus = 256;
    if (hipGetDevice(&dev) == hipSuccess) (void)hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev);
    long long slots = 2ll * cus / pairs;          // two workgroups per CU
    if (slots < 1) slots = 1;
    if (slots > stages) slots = stages;
    return (int)slots;
}

int pick_g(int blocks, int K16, int max_kb) {   // largest G in {4, 2, 1} that divides the block count and fits the panel
    for (int g = 4; g >= 1; g >>= 1)
        if (blocks % g == 0 && g * K16 <= max_kb) return g;
    return 0;
}

}  // namespace

bool k2_supported(const Geom& g, int pass) {
    if (g.dtype != MI3D_BF16 || g.kD != 2 || g.kH != 2 || g.kW != 2) return false;
    if (g.sD != 2 || g.sH != 2 || g.sW != 2 || g.pD || g.pH || g.pW) return false;
    if ((g.D | g.H | g.W) & 1) return false;
    if (g.Cin % 32 || g.Cout % 64) return false;   // k-steps come in fours (the register ring); 64-cout blocks (weight gradient)
    if ((long long)g.N * g.Do * g.Ho * g.Wo >= (1ll << 31)) return false;   // 32-bit voxel arithmetic
    if (pass == MI3D_PASS_WGRAD) return true;
    if (pass == MI3D_PASS_FWD) return pick_g(g.Cout / 32, g.Cin / 2, 128) > 0;
    return pick_g(g.Cin / 4, g.Cout / 16, 64) > 0;
}

size_t k2_workspace_bytes(const Geom& g, int pass) {
    if (!k2_supported(g, pass)) return 0;
    if (pass == MI3D_PASS_WGRAD) return (size_t)k2_wgrad_slots(g) * g.w_elems() * sizeof(float);
    return (((size_t)g.w_elems() * 2 + 255) & ~(size_t)255) + 2048;
}

static int k2_wgrad(const Geom& g, const void* x, const void* dy, float* dw, void* ws, hipStream_t s) {
    K2WgParams P;
    P.x = (const uint16_t*)x; P.dy = (const uint16_t*)dy; P.part = (float*)ws;
    P.Ds = g.Do; P.Hs = g.Ho; P.Ws = g.Wo; P.Cs = g.Cout; P.Cb = g.Cin;
    P.xpitch = g.x_pitch ? g.x_pitch : g.Cin; P.xoff = g.x_off;
    P.vox = (int)((long long)g.N * g.Do * g.Ho * g.Wo);
    P.CiT = g.Cin / WCI;
    P.slots = k2_wgrad_slots(g);
    static std::atomic<bool> attr_set{false};   // set once per process; a second thread racing here repeats an idempotent call
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute((const void*)k2_wgrad_kernel, hipFuncAttributeMaxDynamicSharedMemorySize, 2 * W_STAGE);
        if (e != hipSuccess) { note_hip_error(e); return MI3D_ERR_HIP; }
        attr_set = true;
    }
    k2_wgrad_kernel<<<dim3((unsigned)P.slots, (unsigned)((g.Cout / WCO) * P.CiT)), 256, 2 * W_STAGE, s>>>(P);
    int st = check_launch();
    if (st) return st;
    const long long n = g.w_elems();
    return reduce_partials((const float*)ws, dw, n, P.slots, s);
}

int k2_conv(const Geom& g, int pass, const void* a, const void* w, void* out, void* ws, size_t ws_bytes, hipStream_t s) {
    if (!k2_supported(g, pass)) return MI3D_ERR_UNSUPPORTED;
    if (ws_bytes < k2_workspace_bytes(g, pass)) return MI3D_ERR_WORKSPACE;
    if (pass == MI3D_PASS_WGRAD) return k2_wgrad(g, a, w, (float*)out, ws, s);   // (x, dy, dw)
    const int mode = pass == MI3D_PASS_FWD ? 0 : 1;
    const long long total = g.w_elems();
    k2_pack_kernel<<<(unsigned)((total + 255) / 256), 256, 0, s>>>((const uint16_t*)w, (uint16_t*)ws, g.Cin, g.Cout, mode);
    int st = check_launch();
    if (st) return st;
    K2Params P;
    P.in = (const uint16_t*)a; P.wpack = (const uint16_t*)ws; P.out = (uint16_t*)out;
    P.dump = (uint16_t*)((char*)ws + (((size_t)g.w_elems() * 2 + 255) & ~(size_t)255));
    P.N = g.N; P.Ds = g.Do; P.Hs = g.Ho; P.Ws = g.Wo; P.Cs = g.Cout; P.Cb = g.Cin;
    P.pb = g.x_pitch ? g.x_pitch : g.Cin; P.ob = g.x_off;
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
    // scatter with 32 big-volume channels and a panel per kd: whole voxels per store instruction through LDS
    const bool rows = mode == 1 && G == 4 && g.Cin == 32;
    const size_t lds = (size_t)G * P.K16 * 1024 + (rows ? 4 * K2_STG : 0);
    static std::atomic<bool> attr_set{false};   // set once per process; a second thread racing here repeats an idempotent call
    if (!attr_set) {
        hipError_t e = hipSuccess;
        const void* fns0[3] = {(const void*)k2_kernel<0, 1>, (const void*)k2_kernel<0, 2>, (const void*)k2_kernel<0, 4>};
        const void* fns1[4] = {(const void*)k2_kernel<1, 1>, (const void*)k2_kernel<1, 2>, (const void*)k2_kernel<1, 4>, (const void*)k2_kernel<1, 4, true>};
        for (int i = 0; i < 3 && e == hipSuccess; ++i) e = hipFuncSetAttribute(fns0[i], hipFuncAttributeMaxDynamicSharedMemorySize, 128 * 1024);
        for (int i = 0; i < 4 && e == hipSuccess; ++i) e = hipFuncSetAttribute(fns1[i], hipFuncAttributeMaxDynamicSharedMemorySize, 64 * 1024 + 4 * K2_STG);
        if (e != hipSuccess) { note_hip_error(e); return MI3D_ERR_HIP; }
        attr_set = true;
    }
#define K2_LAUNCH(M, GG) k2_kernel<M, GG><<<(unsigned)P.nwg, 256, lds, s>>>(P)
    if (mode == 0) { if (G == 4) K2_LAUNCH(0, 4); else if (G == 2) K2_LAUNCH(0, 2); else K2_LAUNCH(0, 1); }
    else if (rows) k2_kernel<1, 4, true><<<(unsigned)P.nwg, 256, lds, s>>>(P);
    else { if (G == 4) K2_LAUNCH(1, 4); else if (G == 2) K2_LAUNCH(1, 2); else K2_LAUNCH(1, 1); }
#undef K2_LAUNCH
    return check_launch();
}

}  // namespace mi3d
