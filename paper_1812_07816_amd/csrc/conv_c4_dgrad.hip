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
// walk (16 x 32 patch, plane) units along D; each dy plane patch with halo is
// staged in LDS once and feeds three output planes whose accumulators stay in
// registers.  The pass is bound by its reads of dy, so the staging runs two
// planes ahead of the compute: direct-to-LDS buffer loads fill a ring of three
// stages, and a plane's data has a whole plane step more than the memory
// latency to arrive before anybody waits for it.  LDS holds a patch voxel-major
// (64 bytes per voxel): one load instruction moves 16 neighbouring voxels, 1 KB
// contiguous in memory and in LDS, and a B fragment (16 voxels x 32 couts) is
// again 1 KB contiguous.  (The eight lanes a 16-byte LDS read serves together
// are 64 bytes apart in it, a two-way bank conflict; the pass waits for HBM, not
// for LDS.)
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
constexpr int VB = 64;                             // bytes per staged voxel (32 couts)
constexpr int ROWB = IN_COLS * VB;                 // row pitch in LDS: the patch is a flat list of 18 x 34 voxels
constexpr int NVOX = IN_ROWS * IN_COLS;            // 612
constexpr int NINSTR = (NVOX + 15) / 16;           // load instructions per plane patch, 16 voxels each (39)
constexpr int NLOAD = (NINSTR + 3) / 4;            // per wave (10); instruction k = 4 i + wave
constexpr int STAGE_BYTES = 4 * NLOAD * 1024;      // 40 KB: the last instruction slot is padding
constexpr int NSTAGE = 3;
constexpr unsigned OOB = 0x80000000u;              // buffer offset of a piece that must read as zero
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
// Waits until at most N of this wave's vector-memory operations are outstanding (they complete in issue order) and
// all its LDS reads have returned, then the workgroup barrier.  One asm statement with a memory clobber: the compiler
// moves no LDS access across it.  __syncthreads() would not do here: its workgroup-scope fence makes every
// direct-to-LDS load issued so far complete, including those of the plane two steps ahead.
#define C4D_WAIT_AND_BARRIER(N) asm volatile("s_waitcnt vmcnt(" N ") lgkmcnt(0)\n\ts_barrier" ::: "memory")

// The MFMAs of one staged dy plane for this wave: 10 rows x 3 kw' x 3 kd'.
// kd' = 0 starts a new output plane (its first product accumulates onto zero).
// hook(r) is called once per row: the caller issues one global load there.
template <int PH, class Hook>
__device__ __forceinline__ void plane_compute(f32x4 (&acc)[3][UR], const char* in_lane, const bf16x8 (&wf)[3][3], int kdmask, Hook&& hook) {
    bf16x8 xf[2][3];
#pragma unroll
    for (int kw = 0; kw < 3; ++kw) xf[0][kw] = *(const bf16x8*)(in_lane + kw * VB);
#pragma unroll
    for (int r = 0; r < UR; ++r) {
        if (r + 1 < UR) {
#pragma unroll
            for (int kw = 0; kw < 3; ++kw) xf[(r + 1) & 1][kw] = *(const bf16x8*)(in_lane + (r + 1) * ROWB + kw * VB);
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
    extern __shared__ __attribute__((aligned(16))) char in_lds[];  // ring of NSTAGE stages
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

    // lane (n, g): channels 8g..8g+7 of the voxel in column 16 ch + n (+ kw') of row 8 rh (+ r)
    const int lane_in_off = ((rh * WR) * IN_COLS + ch * 16 + (lane & 15)) * VB + (lane >> 4) * 16;
    const int wave_u = __builtin_amdgcn_readfirstlane(wave);
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

        // staging plan: load i of this wave is instruction 4 i + wave, lane l its 16-byte piece l % 4 of patch voxel
        // 16 (4 i + wave) + l / 4 (row-major over 18 x 34); byte offsets from the plane base, OOB for zero padding
        int goff[NLOAD];
#pragma unroll
        for (int i = 0; i < NLOAD; ++i) {
            const int v = 16 * (4 * i + wave) + (lane >> 2), c = lane & 3;
            const int row = (v * 241) >> 13, col = v - row * IN_COLS;  // v / 34 for v < 700
            const int gh = h0 - P.pH + row, gw = w0 - P.pW + col;
            const bool ok = v < NVOX && gh >= 0 && gh < P.H && gw >= 0 && gw < P.W;
            goff[i] = ok ? ((gh * P.W + gw) * 32 + c * 8) * 2 : (int)OOB;
        }
        const long long plane_elems = (long long)P.H * P.W * 32;
        const uint16_t* dyn = P.dy + (long long)n * P.D * plane_elems;
        uint16_t* dxn = P.dx + (long long)n * P.Do * P.Ho * P.Wo * 4;
        const int nJ = od_end - od_start + 2;

        // A plane outside [0, D) is zero padding: its buffer has zero records, so every piece reads 0 and nothing is
        // fetched; so does a plane past the end of the segment, which nobody reads.  The loads are unconditional.
        __amdgpu_buffer_rsrc_t rsrc = __builtin_amdgcn_make_buffer_rsrc((void*)dyn, 0, 0, 0x00020000);
        const int ip_end = od_start - P.pD + nJ;   // first plane the segment does not read
        auto begin_stage = [&](int ip) {
            const bool inside = ip >= 0 && ip < P.D && ip < ip_end;
            rsrc = __builtin_amdgcn_make_buffer_rsrc((void*)(dyn + (long long)(inside ? ip : 0) * plane_elems), 0,
                                                     inside ? (int)(plane_elems * 2) : 0, 0x00020000);
        };
        auto load_piece = [&](int i, int buf) {
            typedef __attribute__((address_space(3))) void* lds_ptr;
            __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc, (lds_ptr)(in_lds + buf * STAGE_BYTES + (4 * i + wave_u) * 1024), 16, goff[i], 0, 0, 0);
        };

        const int oh0 = h0 + rh * WR, ow = w0 + ch * 16 + (lane & 15);
        const long long row_pitch = (long long)P.Wo * 4;

#pragma unroll
        for (int s = 0; s < 3; ++s)
#pragma unroll
            for (int r = 0; r < UR; ++r) acc[s][r] = f32x4{0.f, 0.f, 0.f, 0.f};

        // the first two planes of the segment; the first one must have arrived, the second may still fly
        begin_stage(od_start - P.pD);
#pragma unroll
        for (int i = 0; i < NLOAD; ++i) load_piece(i, 0);
        begin_stage(od_start + 1 - P.pD);
#pragma unroll
        for (int i = 0; i < NLOAD; ++i) load_piece(i, 1);
        C4D_WAIT_AND_BARRIER("10");

        // Plane step jj computes on dy plane od_start + jj - pD (stage sq % 3), completes output plane
        // od_start + jj - 2 and issues the loads of the plane two steps ahead into the stage that was read one
        // step ago (every wave has passed the barrier behind that step).  At the end of the step the loads issued
        // one step ago must be complete; younger than they are at most this step's ten loads and two stores.
#define C4D_STAGE(PHASE)                                                                        \
        {                                                                                       \
            const int j_ = od_start + jj;                                                       \
            begin_stage(j_ + 2 - P.pD);                                                         \
            const int cur_ = sq % NSTAGE, fill_ = (sq + 2) % NSTAGE;                            \
            int kdmask_ = 0;                                                                    \
            for (int kd_ = 0; kd_ < 3; ++kd_)                                                   \
                if (jj - kd_ >= 0 && jj - kd_ < nJ - 2) kdmask_ |= 1 << kd_;                    \
            plane_compute<PHASE>(acc, in_lds + cur_ * STAGE_BYTES + lane_in_off, wf, kdmask_,   \
                                 [&](int r) { load_piece(r, fill_); });                         \
            store_plane(acc[(PHASE + 1) % 3], dxn + (((long long)(j_ - 2) * P.Ho + oh0) * P.Wo + ow) * 4, \
                        row_pitch, lane, jj >= 2 && ow < P.Wo, P.Ho - oh0, P.dump + lane * 4);  \
            ++sq;                                                                               \
            C4D_WAIT_AND_BARRIER("12");                                                         \
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
    // a staged plane is addressed through a buffer resource with 32-bit byte offsets; 2^31 marks padding
    if ((long long)g.Ho * g.Wo * 64 >= (1ll << 31)) return false;
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
    static std::atomic<bool> attr_set{false};   // set once per process; a second thread racing here repeats an idempotent call
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute((const void*)c4_dgrad_kernel, hipFuncAttributeMaxDynamicSharedMemorySize, NSTAGE * STAGE_BYTES);
        if (e != hipSuccess) { note_hip_error(e); return MI3D_ERR_HIP; }
        attr_set = true;
    }
    c4_dgrad_kernel<<<(unsigned)nwg, 256, NSTAGE * STAGE_BYTES, s>>>(P);
    return check_launch();
}

}  // namespace mi3d
