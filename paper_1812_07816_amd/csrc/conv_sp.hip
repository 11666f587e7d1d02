// Plane-streaming implicit-GEMM convolution for 3x3x3 / stride 1 layers with
// 32 input channels per stage on bf16 MFMA (v_mfma_f32_32x32x16_bf16), fp32
// accumulation.  Serves the forward pass and, with flipped and role-swapped
// weights, the stride-1 data gradient of the feature-map layers of Section 3.1.
//
// Work decomposition
//   column  = (n, cout tile of 32, 16-row x 32-col patch of the output plane)
//   unit    = (column, output plane od); units are dealt to workgroups as
//             contiguous, balanced ranges, so a workgroup walks along D.
//   A workgroup (4 waves) stages ONE input plane patch with halo (18 x 34
//   voxels x 32 ch) in LDS at a time.  That plane feeds the three output
//   planes od = ip + pD - kd; each wave keeps 3 planes x 4 rows of 32x32
//   accumulators in registers, so an input fragment read once from LDS is
//   used by up to 9 (kd, kh) taps and a weight fragment by 4 rows.
//   MFMA roles: A = weights (M = 32 couts), B = input (N = 32 voxels along W),
//   so each lane ends up with 4 consecutive couts of one voxel (8-byte store).
#include "mi3d_internal.h"

namespace mi3d {
namespace {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;

constexpr int TH = 16, TW = 32, RH = 4;            // output patch per workgroup, rows per wave
constexpr int IN_ROWS = TH + 2, IN_COLS = TW + 2;  // with halo
constexpr int COLS = 35;                           // padded row pitch (voxels) in LDS
constexpr int NV = IN_ROWS * COLS;                 // voxels per 8-channel slab (630: 630 % 8 == 6)
constexpr int STAGE_BYTES = 4 * NV * 16;           // 4 slabs of 8 channels, 16 B per voxel
constexpr int W_BYTES = 27 * 2 * 64 * 16;          // 27 taps x 2 k16 steps x 1 KB fragments
constexpr int NLOAD = (IN_ROWS * IN_COLS * 4 + 255) / 256;  // 16-byte loads per thread per plane

struct SpParams {
    const uint16_t* x;
    const uint16_t* wpack;  // [cout tile][cin chunk][kw][kd][kh][k16][lane][8]
    uint16_t* y;
    int N, D, H, W, Cin, Cout, Do, Ho, Wo, pD, pH, pW;
    int HT, WT, CT;         // tiles per plane, cout tiles
    long long units;        // N*CT*HT*WT*Do
    int nwg;
};

__device__ __forceinline__ f32x16 mfma(bf16x8 a, bf16x8 b, f32x16 c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}

template <int PH>
__device__ __forceinline__ void plane_compute(f32x16 (&acc)[3][RH], const char* in_lds, const char* w_lds, int kdmask,
                                              int lane, int wave) {
    const int row0 = wave * RH;
#pragma unroll
    for (int kw = 0; kw < 3; ++kw) {
#pragma unroll
        for (int kk = 0; kk < 2; ++kk) {
            bf16x8 xin[RH + 2];
            const int c = 2 * kk + (lane >> 5);
#pragma unroll
            for (int r = 0; r < RH + 2; ++r)
                xin[r] = *(const bf16x8*)(in_lds + (c * NV + (row0 + r) * COLS + (lane & 31) + kw) * 16);
#pragma unroll
            for (int kd = 0; kd < 3; ++kd) {
                if (kdmask & (1 << kd)) {
#pragma unroll
                    for (int kh = 0; kh < 3; ++kh) {
                        bf16x8 wf = *(const bf16x8*)(w_lds + ((((kw * 3 + kd) * 3 + kh) * 2 + kk) * 64 + lane) * 16);
#pragma unroll
                        for (int r = 0; r < RH; ++r)
                            acc[(PH + 3 - kd) % 3][r] = mfma(wf, xin[r + kh], acc[(PH + 3 - kd) % 3][r]);
                    }
                }
            }
        }
    }
}

__device__ __forceinline__ uint32_t pack2(float a, float b) {
    return (uint32_t)f32_to_bf16_rne(a) | ((uint32_t)f32_to_bf16_rne(b) << 16);
}

__device__ __forceinline__ void store_rows(f32x16 (&a)[RH], uint16_t* yplane, int oh0, int ow, int Ho, int Wo, int Cout,
                                           int co0, int lane) {
#pragma unroll
    for (int r = 0; r < RH; ++r) {
        int oh = oh0 + r;
        if (oh < Ho && ow < Wo) {
            uint16_t* p = yplane + ((long long)oh * Wo + ow) * Cout + co0 + 4 * (lane >> 5);
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                uint2 v;
                v.x = pack2(a[r][4 * g + 0], a[r][4 * g + 1]);
                v.y = pack2(a[r][4 * g + 2], a[r][4 * g + 3]);
                *(uint2*)(p + 8 * g) = v;
            }
        }
#pragma unroll
        for (int i = 0; i < 16; ++i) a[r][i] = 0.f;
    }
}

__global__ void __launch_bounds__(256, 1) sp_conv_kernel(SpParams P) {
    extern __shared__ __attribute__((aligned(16))) char lds[];
    char* w_lds = lds;
    char* in_lds = lds + W_BYTES;  // two stages

    const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
    // XCD-aware placement: hardware deals consecutive workgroup ids round-robin
    // over the 8 XCDs; give each XCD one contiguous range of units so that
    // neighbouring patches (which share halos) meet in the same L2.
    int g = blockIdx.x;
    if ((P.nwg & 7) == 0) g = (g & 7) * (P.nwg >> 3) + (g >> 3);
    long long u0 = P.units * g / P.nwg, u1 = P.units * (g + 1) / P.nwg;

    // per-thread load plan for one plane patch (does not depend on the plane)
    int lds_off[NLOAD], rowcol[NLOAD];
#pragma unroll
    for (int i = 0; i < NLOAD; ++i) {
        int q = t + 256 * i;
        int v = q >> 2, c = q & 3;
        int row = v / IN_COLS, col = v - row * IN_COLS;
        lds_off[i] = (c * NV + row * COLS + col) * 16;
        rowcol[i] = (q < IN_ROWS * IN_COLS * 4) ? ((row << 16) | (col << 4) | (c << 1) | 1) : 0;
    }

    f32x16 acc[3][RH];
#pragma unroll
    for (int s = 0; s < 3; ++s)
#pragma unroll
        for (int r = 0; r < RH; ++r)
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[s][r][i] = 0.f;

    int cur_ct = -1;
    while (u0 < u1) {
        long long column = u0 / P.Do;
        int od_start = (int)(u0 - column * P.Do);
        int od_end = od_start + (int)((u1 - u0) < (long long)(P.Do - od_start) ? (u1 - u0) : (long long)(P.Do - od_start));
        u0 += od_end - od_start;
        int wt = (int)(column % P.WT); column /= P.WT;
        int ht = (int)(column % P.HT); column /= P.HT;
        int ct = (int)(column % P.CT);
        int n = (int)(column / P.CT);
        const int h0 = ht * TH, w0 = wt * TW;

        if (ct != cur_ct) {  // (re)load the weights of this cout tile; previous readers passed a barrier
            const uint4* src = (const uint4*)(P.wpack + (long long)ct * (W_BYTES / 2));
            for (int i = t; i < W_BYTES / 16; i += 256) ((uint4*)w_lds)[i] = src[i];
            cur_ct = ct;
        }
        // global offsets (elements) of this patch relative to the plane base
        int goff[NLOAD];
        unsigned valid = 0;
#pragma unroll
        for (int i = 0; i < NLOAD; ++i) {
            int row = rowcol[i] >> 16, col = (rowcol[i] >> 4) & 0xfff, c = (rowcol[i] >> 1) & 7;
            int gh = h0 - P.pH + row, gw = w0 - P.pW + col;
            bool ok = (rowcol[i] & 1) && gh >= 0 && gh < P.H && gw >= 0 && gw < P.W;
            goff[i] = ok ? (gh * P.W + gw) * P.Cin + c * 8 : 0;
            valid |= (ok ? 1u : 0u) << i;
        }
        const long long plane_elems = (long long)P.H * P.W * P.Cin;
        const uint16_t* xn = P.x + (long long)n * P.D * plane_elems;
        uint16_t* yn = P.y + (long long)n * P.Do * P.Ho * P.Wo * P.Cout;
        const int nJ = od_end - od_start + 2;
        uint4 pre[NLOAD];

        auto load_plane = [&](int ip) {
            const uint16_t* base = xn + (long long)ip * plane_elems;
#pragma unroll
            for (int i = 0; i < NLOAD; ++i) {
                uint4 z = {0, 0, 0, 0};
                pre[i] = ((valid >> i) & 1) ? *(const uint4*)(base + goff[i]) : z;
            }
        };
        auto write_plane = [&](int buf) {
#pragma unroll
            for (int i = 0; i < NLOAD; ++i)
                if (rowcol[i] & 1) *(uint4*)(in_lds + buf * STAGE_BYTES + lds_off[i]) = pre[i];
        };

        {
            int ip = od_start - P.pD;
            if (ip >= 0 && ip < P.D) { load_plane(ip); write_plane(0); }
        }
        __syncthreads();

#define SP_STEP(PHASE, JJ)                                                                      \
        {                                                                                       \
            const int jj_ = (JJ);                                                               \
            const int j_ = od_start + jj_;                                                      \
            const int ip_ = j_ - P.pD;                                                          \
            const bool valid_ = ip_ >= 0 && ip_ < P.D;                                          \
            const bool validn_ = (jj_ + 1 < nJ) && (ip_ + 1 >= 0) && (ip_ + 1 < P.D);           \
            if (validn_) load_plane(ip_ + 1);                                                   \
            if (valid_) {                                                                       \
                int m_ = 0;                                                                     \
                for (int kd = 0; kd < 3; ++kd)                                                  \
                    if (j_ - kd >= od_start && j_ - kd < od_end) m_ |= 1 << kd;                 \
                plane_compute<PHASE>(acc, in_lds + (jj_ & 1) * STAGE_BYTES, w_lds, m_, lane, wave); \
            }                                                                                   \
            if (validn_) write_plane((jj_ + 1) & 1);                                            \
            __syncthreads();                                                                    \
            if (jj_ >= 2) {                                                                     \
                const int od_ = j_ - 2;                                                         \
                store_rows(acc[((PHASE) + 1) % 3], yn + (long long)od_ * P.Ho * P.Wo * P.Cout,  \
                           h0 + wave * RH, w0 + (lane & 31), P.Ho, P.Wo, P.Cout, ct * 32, lane); \
            }                                                                                   \
        }
        for (int jj = 0; jj < nJ; jj += 3) {
            SP_STEP(0, jj)
            if (jj + 1 < nJ) SP_STEP(1, jj + 1)
            if (jj + 2 < nJ) SP_STEP(2, jj + 2)
        }
#undef SP_STEP
    }
}

// Rearranges [Cout][3][3][3][Cin] weights into per-lane MFMA A fragments.
// flip = 0: forward.  flip = 1: stride-1 data gradient, i.e. a forward
// convolution over dy whose weights are w'[ci][t'][co] = w[co][2 - t'][ci].
__global__ void __launch_bounds__(256) sp_pack_weights_kernel(const uint16_t* __restrict__ w, uint16_t* __restrict__ wpack,
                                                              int Cin, int Cout, int flip) {
    // packed "output" channels / "input" channels of the convolution being run
    const int Co = flip ? Cin : Cout, Ci = flip ? Cout : Cin;
    long long total = 27ll * Co * Ci;
    long long idx = (long long)blockIdx.x * 256 + threadIdx.x;
    if (idx >= total) return;
    int j = (int)(idx & 7);
    long long r = idx >> 3;
    int lane = (int)(r & 63); r >>= 6;
    int kk = (int)(r & 1); r >>= 1;
    int kh = (int)(r % 3); r /= 3;
    int kd = (int)(r % 3); r /= 3;
    int kw = (int)(r % 3); r /= 3;
    int chunks = Ci / 32;
    int chunk = (int)(r % chunks);
    int ct = (int)(r / chunks);
    int co = ct * 32 + (lane & 31);
    int ci = chunk * 32 + kk * 16 + 8 * (lane >> 5) + j;
    uint16_t v;
    if (!flip) v = w[((((long long)co * 3 + kd) * 3 + kh) * 3 + kw) * Cin + ci];
    else v = w[((((long long)ci * 3 + (2 - kd)) * 3 + (2 - kh)) * 3 + (2 - kw)) * Cin + co];
    wpack[idx] = v;
}

}  // namespace

bool sp_supported(const Geom& g, int pass) {
    if (g.dtype != MI3D_BF16 || g.kD != 3 || g.kH != 3 || g.kW != 3) return false;
    if (g.sD != 1 || g.sH != 1 || g.sW != 1) return false;
    if (g.pD > 2 || g.pH > 2 || g.pW > 2) return false;
    if (pass == MI3D_PASS_FWD) return g.Cin == 32 && g.Cout % 32 == 0;
    if (pass == MI3D_PASS_DGRAD) return g.Cout == 32 && g.Cin % 32 == 0;
    return false;
}

size_t sp_workspace_bytes(const Geom& g, int pass) {
    if (!sp_supported(g, pass)) return 0;
    return (size_t)g.w_elems() * 2;
}

// in: activations read (x for fwd, dy for dgrad); out: y or dx
int sp_conv(const Geom& g, int pass, const void* in, const void* w, void* out, void* ws, size_t ws_bytes, hipStream_t s) {
    if (ws_bytes < sp_workspace_bytes(g, pass)) return MI3D_ERR_WORKSPACE;
    const bool flip = pass == MI3D_PASS_DGRAD;
    long long total = g.w_elems();
    sp_pack_weights_kernel<<<(unsigned)((total + 255) / 256), 256, 0, s>>>((const uint16_t*)w, (uint16_t*)ws, g.Cin, g.Cout, flip ? 1 : 0);
    int st = check_launch();
    if (st) return st;
    SpParams P;
    P.x = (const uint16_t*)in;
    P.wpack = (const uint16_t*)ws;
    P.y = (uint16_t*)out;
    P.N = g.N;
    if (!flip) {
        P.D = g.D; P.H = g.H; P.W = g.W; P.Cin = g.Cin; P.Cout = g.Cout;
        P.Do = g.Do; P.Ho = g.Ho; P.Wo = g.Wo; P.pD = g.pD; P.pH = g.pH; P.pW = g.pW;
    } else {  // convolution over dy producing dx, pad' = k - 1 - p
        P.D = g.Do; P.H = g.Ho; P.W = g.Wo; P.Cin = g.Cout; P.Cout = g.Cin;
        P.Do = g.D; P.Ho = g.H; P.Wo = g.W; P.pD = 2 - g.pD; P.pH = 2 - g.pH; P.pW = 2 - g.pW;
    }
    P.HT = (P.Ho + TH - 1) / TH;
    P.WT = (P.Wo + TW - 1) / TW;
    P.CT = P.Cout / 32;
    P.units = (long long)P.N * P.CT * P.HT * P.WT * P.Do;
    int dev = 0, cus = 256;
    if (hipGetDevice(&dev) == hipSuccess) (void)hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev);
    long long nwg = cus;
    if (nwg > P.units) nwg = P.units;
    P.nwg = (int)nwg;
    size_t lds = W_BYTES + 2 * STAGE_BYTES;
    static bool attr_set = false;
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute((const void*)sp_conv_kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) { note_hip_error(e); return MI3D_ERR_HIP; }
        attr_set = true;
    }
    sp_conv_kernel<<<(unsigned)nwg, 256, lds, s>>>(P);
    return check_launch();
}

}  // namespace mi3d
