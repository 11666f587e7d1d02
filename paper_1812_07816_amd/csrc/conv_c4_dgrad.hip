// Data gradient of the network's first layer (3x3x3 / stride 1, 4 input
// channels, 32 output channels): dx[v, ci] = sum_{t, co} dy[v + p - t, co] w[co, t, ci],
// i.e. a convolution over dy with flipped taps that produces only 4 channels.
//
// The pass reads dy once (32 channels) and writes 4 channels, so it is bound
// by HBM reads; a 32-wide MFMA n or m dimension padded from 4 channels would
// waste 7/8 of the matrix work instead.  Here the (kh, ci) pairs are folded
// into the MFMA m dimension (12 of 16 rows used) of v_mfma_f32_16x16x32_bf16:
//   A = weights of one (kd, kw) tap pair, rows m = 4 kh + ci, k = 32 couts
//   B = 16 dy voxels of one staged row, shifted along W by kw through the
//       lane's own LDS address, k = 32 couts
//   C = for every dy row r: U[r][kh][ci][col], the part of output row r - kh
//       that comes through tap row kh.
// One accumulator per dy row collects all 9 (kd, kw) products; the three kh
// parts of an output row then sit in three different accumulators and three
// different 16-lane groups.  A select per lane group and a transposing
// butterfly over the lane groups (v_permlane32_swap, v_permlane16_swap) sums
// them, leaving four finished output rows in the four lane groups.
//
// Work decomposition as in the plane-streaming kernel: persistent workgroups
// walk (16 x 32 patch, plane) units along D, one dy plane patch with halo is
// staged in LDS at a time (double buffered) and feeds three output planes
// whose accumulators stay in registers.
#include "mi3d_internal.h"

namespace mi3d {
namespace {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float f32x4;
typedef __attribute__((__vector_size__(2 * sizeof(float)))) float f32x2;
typedef __attribute__((__vector_size__(2 * sizeof(__bf16)))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(2))) unsigned u32x2;

constexpr int TH = 16, TW = 32;
constexpr int WR = 8, UR = WR + 2;                 // output rows per wave, dy rows they meet
constexpr int IN_ROWS = TH + 2, IN_COLS = TW + 2;  // staged patch with halo
constexpr int COLS = 35;                           // row pitch (voxels) in LDS
constexpr int NV = IN_ROWS * COLS;                 // voxels per 8-channel slab
constexpr int STAGE_BYTES = 4 * NV * 16;           // [8-channel slab][row][col] x 16 B
constexpr int NPIECE = IN_ROWS * IN_COLS * 4;      // 16-byte pieces per plane patch
constexpr int NLOAD = (NPIECE + 255) / 256;        // 10 per thread
static_assert(NLOAD == UR, "one global load per dy row step");

struct C4DgParams {
    const uint16_t* dy;
    const uint16_t* wpack;  // [kd'][kw'][lane][8], flipped taps
    uint16_t* dx;
    uint16_t* dump;         // 512 B that masked store lanes write to instead of dx
    int N, D, H, W;         // extents of dy (the tensor read)
    int Do, Ho, Wo;         // extents of dx (the tensor written)
    int pD, pH, pW;         // padding of the equivalent forward convolution over dy: 2 - p
    int HT, WT;
    long long units;        // N*HT*WT*Do
    int nwg;
};

#define C4D_FENCE() __builtin_amdgcn_sched_barrier(0)

// The MFMAs of one staged dy plane for this wave: 10 rows x 3 kw' x 3 kd'.
// kd' = 0 starts a new output plane (its first product accumulates onto zero).
// hook(r) is called once per row: the caller issues one global load there.
template <int PH, class Hook>
__device__ __forceinline__ void plane_compute(f32x4 (&acc)[3][UR], const char* in_lane, const bf16x8 (&wf)[3][3], int kdmask, Hook&& hook) {
    bf16x8 xf[2][3];
#pragma unroll
    for (int kw = 0; kw < 3; ++kw) xf[0][kw] = *(const bf16x8*)(in_lane + kw * 16);
#pragma unroll
    for (int r = 0; r < UR; ++r) {
        if (r + 1 < UR) {
#pragma unroll
            for (int kw = 0; kw < 3; ++kw) xf[(r + 1) & 1][kw] = *(const bf16x8*)(in_lane + ((r + 1) * COLS + kw) * 16);
        }
#pragma unroll
        for (int kd = 2; kd >= 0; --kd) {
            if (!(kdmask & (1 << kd))) continue;
            f32x4& a = acc[(PH + 3 - kd) % 3][r];
#pragma unroll
            for (int kw = 0; kw < 3; ++kw) {
                if (kd == 0 && kw == 0) {
                    f32x4 z = {0.f, 0.f, 0.f, 0.f};
                    a = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wf[kd][kw], xf[r & 1][kw], z, 0, 0, 0);
                } else {
                    a = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wf[kd][kw], xf[r & 1][kw], a, 0, 0, 0);
                }
            }
        }
        hook(r);
        C4D_FENCE();
    }
}

// Sum of the two results of a lane-group swap.  Each result passes through an empty asm
// statement: adding the two builtin results directly was compiled into an add of the first result
// with itself (hipcc 7.2, seen in the ISA listing).
__device__ __forceinline__ float add_pair(u32x2 s) {
    unsigned r0 = s[0], r1 = s[1];
    asm volatile("" : "+v"(r0), "+v"(r1));
    return __builtin_bit_cast(float, r0) + __builtin_bit_cast(float, r1);
}
__device__ __forceinline__ float swap_add32(float a, float b) {
    return add_pair(__builtin_amdgcn_permlane32_swap(__builtin_bit_cast(unsigned, a), __builtin_bit_cast(unsigned, b), false, false));
}
__device__ __forceinline__ float swap_add16(float a, float b) {
    return add_pair(__builtin_amdgcn_permlane16_swap(__builtin_bit_cast(unsigned, a), __builtin_bit_cast(unsigned, b), false, false));
}

// Finished plane: U[r] lane group g holds the tap-row-g part of output row r - g.
// Output row i = sum over g of U[i + g] in lane group g (group 3 is all zero:
// its weight rows are padding).  Four rows at a time: after the butterfly lane
// group g holds output row 4 q + g, each lane the 4 channels of one voxel.
// Stores are unconditional (masked lanes write to the dump area): behind a branch the compiler cannot count them
// and makes the LDS write that follows wait for vmcnt(0), i.e. for the stores themselves.
__device__ __forceinline__ void store_plane(const f32x4 (&U)[UR], uint16_t* p, long long row_pitch, int lane, bool col_ok, int rows_left, uint16_t* dump) {
    const int g = lane >> 4;
#pragma unroll
    for (int q = 0; q < WR / 4; ++q) {
        f32x4 V[4];
#pragma unroll
        for (int a = 0; a < 4; ++a)
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const int i = 4 * q + a;
                V[a][v] = g == 0 ? U[i][v] : (g == 1 ? U[i + 1][v] : U[i + 2][v]);
            }
        float tot[4];
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            // halves: lane groups (0+2, 1+3) of rows (0, 2) and of rows (1, 3); then odd/even groups
            const float s02 = swap_add32(V[0][v], V[2][v]);
            const float s13 = swap_add32(V[1][v], V[3][v]);
            tot[v] = swap_add16(s02, s13);
        }
        f32x2 lo = {tot[0], tot[1]}, hi = {tot[2], tot[3]};
        uint2 o;
        o.x = __builtin_bit_cast(uint32_t, __builtin_convertvector(lo, bf16x2));
        o.y = __builtin_bit_cast(uint32_t, __builtin_convertvector(hi, bf16x2));
        *(uint2*)((col_ok && 4 * q + g < rows_left) ? p + (4 * q + g) * row_pitch : dump) = o;
    }
}

__global__ void __launch_bounds__(256, 1) c4_dgrad_kernel(C4DgParams P) {
    extern __shared__ __attribute__((aligned(16))) char in_lds[];  // 2 stages
    const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
    const int rh = wave >> 1, ch = wave & 1;  // half of the patch rows, half of its columns
    int gidx = blockIdx.x;
    if ((P.nwg & 7) == 0) gidx = (gidx & 7) * (P.nwg >> 3) + (gidx >> 3);  // one contiguous unit range per XCD
    long long u0 = P.units * gidx / P.nwg, u1 = P.units * (gidx + 1) / P.nwg;

    // weights stay in registers: 9 fragments of 16 (kh, ci) rows x 32 couts
    bf16x8 wf[3][3];
#pragma unroll
    for (int kd = 0; kd < 3; ++kd)
#pragma unroll
        for (int kw = 0; kw < 3; ++kw) wf[kd][kw] = *((const bf16x8*)P.wpack + (kd * 3 + kw) * 64 + lane);

    int lds_off[NLOAD];
#pragma unroll
    for (int i = 0; i < NLOAD; ++i) {
        const int q = t + 256 * i;
        const int v = q >> 2, c = q & 3;
        const int row = (v * 241) >> 13, col = v - row * IN_COLS;  // v / 34 for v < 700
        lds_off[i] = (c * NV + row * COLS + col) * 16;
    }
    // lane (n, g): channels 8g..8g+7 of the voxel in column 16 ch + n (+ kw') of row 8 rh (+ r)
    const int lane_in_off = ((lane >> 4) * NV + rh * WR * COLS + ch * 16 + (lane & 15)) * 16;
    f32x4 acc[3][UR];

    while (u0 < u1) {
        long long column = u0 / P.Do;
        const int od_start = (int)(u0 - column * P.Do);
        const int od_end = od_start + (int)((u1 - u0) < (long long)(P.Do - od_start) ? (u1 - u0) : (long long)(P.Do - od_start));
        u0 += od_end - od_start;
        const int wt = (int)(column % P.WT); column /= P.WT;
        const int ht = (int)(column % P.HT);
        const int n = (int)(column / P.HT);
        const int h0 = ht * TH, w0 = wt * TW;

        int goff[NLOAD];
        unsigned valid = 0;
#pragma unroll
        for (int i = 0; i < NLOAD; ++i) {
            const int q = t + 256 * i;
            const int v = q >> 2, c = q & 3;
            const int row = (v * 241) >> 13, col = v - row * IN_COLS;
            const int gh = h0 - P.pH + row, gw = w0 - P.pW + col;
            const bool ok = q < NPIECE && gh >= 0 && gh < P.H && gw >= 0 && gw < P.W;
            goff[i] = ok ? (gh * P.W + gw) * 32 + c * 8 : 0;
            valid |= (ok ? 1u : 0u) << i;
        }
        const long long plane_elems = (long long)P.H * P.W * 32;
        const uint16_t* dyn = P.dy + (long long)n * P.D * plane_elems;
        uint16_t* dxn = P.dx + (long long)n * P.Do * P.Ho * P.Wo * 4;
        const int nJ = od_end - od_start + 2;

        // loads are unconditional (masked pieces read element 0 of a valid plane) and zeroed when
        // they are written to LDS, so nothing waits for them before the MFMA work
        uint4 pre[NLOAD];
        unsigned pre_mask = 0;
        const uint16_t* pre_base = dyn;
        auto begin_stage = [&](int ip) {
            const bool inside = ip >= 0 && ip < P.D;
            pre_base = dyn + (long long)(inside ? ip : 0) * plane_elems;
            pre_mask = inside ? valid : 0u;
        };
        auto load_piece = [&](int i) { pre[i] = *(const uint4*)(pre_base + goff[i]); };
        auto write_stage = [&](int buf) {
            char* dst = in_lds + buf * STAGE_BYTES;
#pragma unroll
            for (int i = 0; i < NLOAD; ++i) {
                const bool ok = (pre_mask >> i) & 1;
                uint4 v;
                v.x = ok ? pre[i].x : 0u;
                v.y = ok ? pre[i].y : 0u;
                v.z = ok ? pre[i].z : 0u;
                v.w = ok ? pre[i].w : 0u;
                if (t + 256 * i < NPIECE) *(uint4*)(dst + lds_off[i]) = v;
            }
        };

        const int oh0 = h0 + rh * WR, ow = w0 + ch * 16 + (lane & 15);
        const long long row_pitch = (long long)P.Wo * 4;

#pragma unroll
        for (int s = 0; s < 3; ++s)
#pragma unroll
            for (int r = 0; r < UR; ++r) acc[s][r] = f32x4{0.f, 0.f, 0.f, 0.f};

        begin_stage(od_start - P.pD);
#pragma unroll
        for (int i = 0; i < NLOAD; ++i) load_piece(i);
        write_stage(0);
        __syncthreads();

        // plane step jj stages dy plane od_start + jj - pD and completes output plane od_start + jj - 2
#define C4D_STAGE(PHASE)                                                                        \
        {                                                                                       \
            const int j_ = od_start + jj;                                                       \
            begin_stage(j_ + 1 - P.pD);                                                         \
            int kdmask_ = 0;                                                                    \
            for (int kd_ = 0; kd_ < 3; ++kd_)                                                   \
                if (jj - kd_ >= 0 && jj - kd_ < nJ - 2) kdmask_ |= 1 << kd_;                    \
            plane_compute<PHASE>(acc, in_lds + (sq & 1) * STAGE_BYTES + lane_in_off, wf, kdmask_, \
                                 [&](int r) { load_piece(r); });                                \
            store_plane(acc[(PHASE + 1) % 3], dxn + (((long long)(j_ - 2) * P.Ho + oh0) * P.Wo + ow) * 4, \
                        row_pitch, lane, jj >= 2 && ow < P.Wo, P.Ho - oh0, P.dump + lane * 4);  \
            write_stage((sq + 1) & 1);                                                          \
            ++sq;                                                                               \
            __syncthreads();                                                                    \
        }
        int sq = 0;
        for (int jj = 0;;) {
            C4D_STAGE(0)
            if (++jj >= nJ) break;
            C4D_STAGE(1)
            if (++jj >= nJ) break;
            C4D_STAGE(2)
            if (++jj >= nJ) break;
        }
#undef C4D_STAGE
    }
}

// [32][3][3][3][4] weights -> [kd'][kw'][lane][8] A fragments of the flipped convolution:
// lane (m, g): row m = 4 kh' + ci (rows 12..15 zero), k = 8 g + j = cout
__global__ void __launch_bounds__(256) c4_dgrad_pack_kernel(const uint16_t* __restrict__ w, uint16_t* __restrict__ wpack) {
    const int idx = blockIdx.x * 256 + threadIdx.x;
    if (idx >= 9 * 512) return;
    const int j = idx & 7, lane = (idx >> 3) & 63, tap = idx >> 9;
    const int kd = tap / 3, kw = tap % 3;
    const int m = lane & 15, g = lane >> 4;
    const int kh = m >> 2, ci = m & 3, co = 8 * g + j;
    wpack[idx] = kh < 3 ? w[(((co * 3 + (2 - kd)) * 3 + (2 - kh)) * 3 + (2 - kw)) * 4 + ci] : (uint16_t)0;
}

}  // namespace

bool c4_dgrad_supported(const Geom& g) {
    if (g.dtype != MI3D_BF16 || g.kD != 3 || g.kH != 3 || g.kW != 3) return false;
    if (g.sD != 1 || g.sH != 1 || g.sW != 1) return false;
    if (g.pD > 2 || g.pH > 2 || g.pW > 2) return false;
    return g.Cin == 4 && g.Cout == 32;
}

size_t c4_dgrad_workspace_bytes(const Geom& g) { return c4_dgrad_supported(g) ? 9 * 1024 + 512 : 0; }

int c4_dgrad(const Geom& g, const void* dy, const void* w, void* dx, void* ws, size_t ws_bytes, hipStream_t s) {
    if (ws_bytes < c4_dgrad_workspace_bytes(g)) return MI3D_ERR_WORKSPACE;
    c4_dgrad_pack_kernel<<<18, 256, 0, s>>>((const uint16_t*)w, (uint16_t*)ws);
    int st = check_launch();
    if (st) return st;
    C4DgParams P;
    P.dy = (const uint16_t*)dy; P.wpack = (const uint16_t*)ws; P.dx = (uint16_t*)dx;
    P.dump = (uint16_t*)((char*)ws + 9 * 1024);
    P.N = g.N;
    P.D = g.Do; P.H = g.Ho; P.W = g.Wo;
    P.Do = g.D; P.Ho = g.H; P.Wo = g.W;
    P.pD = 2 - g.pD; P.pH = 2 - g.pH; P.pW = 2 - g.pW;
    P.HT = (P.Ho + TH - 1) / TH;
    P.WT = (P.Wo + TW - 1) / TW;
    P.units = (long long)P.N * P.HT * P.WT * P.Do;
    int dev = 0, cus = 256;
    if (hipGetDevice(&dev) == hipSuccess) (void)hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev);
    long long nwg = cus;
    if (nwg > P.units) nwg = P.units;
    P.nwg = (int)nwg;
    static bool attr_set = false;
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute((const void*)c4_dgrad_kernel, hipFuncAttributeMaxDynamicSharedMemorySize, 2 * STAGE_BYTES);
        if (e != hipSuccess) { note_hip_error(e); return MI3D_ERR_HIP; }
        attr_set = true;
    }
    c4_dgrad_kernel<<<(unsigned)nwg, 256, 2 * STAGE_BYTES, s>>>(P);
    return check_launch();
}

}  // namespace mi3d
