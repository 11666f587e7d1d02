// Weight gradient of the 3x3x3 / stride 2 convolution on bf16 MFMA
// (v_mfma_f32_16x16x32_bf16), fp32 accumulation and fp32 output:
//   dw[co,t,ci] = sum_{n,o} dy[n,o,co] * x[n, 2 o - p + t, ci]
// Same scheme as the stride-1 weight gradient (transposing LDS reads, a
// register window of dy fragments, one (32 cout x 32 cin) pair per workgroup,
// 16x16 quadrant per wave, deterministic slot reduction), with the index maps
// of stride 2: x plane id meets dy plane od through tap kd only when
// id + pD = 2 od + kd, so planes with even id + pD serve taps 0 and 2 and odd
// ones tap 1; the same holds for rows (kh).  The staged x patch (9 x 65
// voxels for 4 x 32 dy voxels) is split by column parity so that the voxels
// 2 j + kw of a fragment are neighbours in LDS.  The x patches, nine tenths
// of the staged bytes, are fetched two planes ahead with direct-to-LDS loads
// into a ring of three stages (voxel-major, 64 bytes per voxel: one load
// instruction moves 16 voxels of one column parity, 64 contiguous bytes
// each); the small dy patches follow one step ahead the same way.  The load
// instructions are written as inline assembly: the compiler makes every
// transposing LDS read wait for all direct-to-LDS loads it knows of, which
// would undo the two-plane lead.
#include "mi3d_internal.h"

namespace mi3d {
namespace {

typedef __attribute__((__vector_size__(4 * sizeof(short)))) short s16x4;
typedef __attribute__((__vector_size__(8 * sizeof(short)))) short s16x8;
typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float f32x4;

constexpr int TH = 4, TW = 32;
constexpr int XR = 2 * TH + 1, XC = 2 * TW + 1;  // 9 x 65
constexpr int XHALF = 33, XPITCH = 2 * XHALF;    // row of the staged patch: even columns, then odd columns
constexpr int XVB = 64;                          // bytes per staged x voxel (32 cins)
constexpr int XPOS = XR * XPITCH;                // voxel positions of a staged patch (594)
constexpr int NXI = (XPOS + 15) / 16;            // load instructions per patch, 16 positions each (38)
constexpr int NX = (NXI + 3) / 4;                // per wave (10); instruction k = 4 i + wave
constexpr int X_BYTES = 4 * NX * 1024;           // 40 KB per stage: the last two instruction slots are padding
constexpr int XSTAGES = 3;
constexpr int DY_SLAB = TH * TW * 32;            // one 16-cout slab of the dy patch
constexpr unsigned OOB = 0x80000000u;            // buffer offset of a piece that must read as zero
// Waits until at most N of this wave's vector-memory operations are outstanding (they complete in issue order) and
// its LDS accesses have finished, then the workgroup barrier; one asm statement with a memory clobber, so the
// compiler moves no LDS access across it.  __syncthreads() would not do: its workgroup-scope fence makes every
// direct-to-LDS load issued so far complete, including those of the plane two steps ahead.
#define WG2_WAIT_AND_BARRIER(N) asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)\n\ts_barrier" ::"n"(N) : "memory")

typedef __attribute__((ext_vector_type(4))) unsigned u32x4;
// buffer resource over `bytes` bytes at p (raw buffer, offsets beyond the range read as zero)
__device__ __forceinline__ u32x4 make_rsrc(const void* p, unsigned bytes) {
    const unsigned long long b = (unsigned long long)p;
    return u32x4{(unsigned)b, (unsigned)(b >> 32) & 0xffffu, bytes, 0x00020000u};
}
// One direct-to-LDS load: lane l moves the 16 bytes at byte offset voff (its own) of the buffer to LDS address
// lds_addr + 16 l (lds_addr uniform).  Counts in vmcnt like any vector-memory load.
__device__ __forceinline__ void dma16(u32x4 rsrc, unsigned lds_addr, int voff) {
    asm volatile("s_mov_b32 m0, %0\n\tbuffer_load_dwordx4 %1, %2, 0 offen lds" ::"s"(lds_addr), "v"(voff), "s"(rsrc) : "memory", "m0");
}

struct Wg2Params {
    const uint16_t* x;
    const uint16_t* dy;
    float* part;
    int N, D, H, W, Cin, Cout, Do, Ho, Wo, pD, pH, pW;
    int HT, WT, CiT, CoT;   // CoT: cout tiles of 32 MB
    long long units;  // per pair: N*HT*WT*D
    int slots;
};

// VB: bytes between neighbouring voxels of the staged operand
template <int VB = 32>
__device__ __forceinline__ bf16x8 tr_frag(const char* p) {
    typedef __attribute__((address_space(3))) s16x4* lptr;
    s16x4 a = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lptr)(p));
    s16x4 b = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lptr)(p + 16 * VB));
    s16x8 c = __builtin_shufflevector(a, b, 0, 1, 2, 3, 4, 5, 6, 7);
    return __builtin_bit_cast(bf16x8, c);
}

__device__ __forceinline__ f32x4 mfma16(bf16x8 a, bf16x8 b, f32x4 c) {
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, c, 0, 0, 0);
}

// One staged x plane.  EVEN: id + pD even, taps kd 0 (dy plane in dy_lane[0]) and kd 2 (dy_lane[1]);
// otherwise tap kd 1 (dy_lane[0]).  x row R meets dy row dr through kh = R - 2 dr.
// MB: 16-cout blocks per wave (consecutive slabs of the dy patch); each x fragment then feeds MB MFMAs.
template <bool EVEN, int MB, class Hook>
__device__ __forceinline__ void plane_step(f32x4 (&acc)[MB][3][3][3], const char* x_lane, const char* const (&dy_lane)[2], Hook&& hook) {
    constexpr int NKD = EVEN ? 2 : 1;
    bf16x8 dyw[NKD][3][MB];  // window over dy rows, slot = dr % 3
#pragma unroll
    for (int k = 0; k < NKD; ++k)
#pragma unroll
        for (int b = 0; b < MB; ++b) dyw[k][0][b] = tr_frag(dy_lane[k] + b * DY_SLAB);
    // x fragments are read three rows ahead of their use (ring of four); left to the compiler every row is
    // read -> wait -> MFMAs, and with 3 to 12 MFMAs per row two rows do not cover the LDS latency
    constexpr int AH = MB == 2 ? 2 : 3;   // (with two cout blocks a row holds twice the MFMAs, and the registers are needed elsewhere)
    bf16x8 xf[AH + 1][3];
    auto load_xrow = [&](int R) {
#pragma unroll
        for (int kw = 0; kw < 3; ++kw) xf[R % (AH + 1)][kw] = tr_frag<XVB>(x_lane + (R * XPITCH + (kw & 1) * XHALF + (kw >> 1)) * XVB);
    };
#pragma unroll
    for (int R = 0; R < AH; ++R) load_xrow(R);
#pragma unroll
    for (int R = 0; R < XR; ++R) {
        if (R + AH < XR) load_xrow(R + AH);
        if ((R & 1) == 0 && R / 2 + 1 < TH) {  // the dy row that the next even x row starts using
#pragma unroll
            for (int k = 0; k < NKD; ++k)
#pragma unroll
                for (int b = 0; b < MB; ++b) dyw[k][(R / 2 + 1) % 3][b] = tr_frag(dy_lane[k] + b * DY_SLAB + (R / 2 + 1) * TW * 32);
        }
#pragma unroll
        for (int kh = 0; kh < 3; ++kh) {
            if (((R - kh) & 1) != 0) continue;
            const int dr = (R - kh) / 2;
            if (R - kh < 0 || dr >= TH) continue;
#pragma unroll
            for (int k = 0; k < NKD; ++k) {
                const int kd = EVEN ? 2 * k : 1;
#pragma unroll
                for (int kw = 0; kw < 3; ++kw)
#pragma unroll
                    for (int b = 0; b < MB; ++b) acc[b][kd][kh][kw] = mfma16(dyw[k][dr % 3][b], xf[R % (AH + 1)][kw], acc[b][kd][kh][kw]);
            }
        }
        hook(R);
        __builtin_amdgcn_sched_barrier(0);
    }
}

// MB = 1: a workgroup serves a (32 cout x 32 cin) pair, a wave a 16 x 16 quadrant.  MB = 2 (Cout % 64 == 0): a
// (64 cout x 32 cin) pair, a wave 32 couts x 16 cins: the x patch, nine tenths of the staged bytes, is fetched once
// per 64 couts instead of once per 32, and the kernel is bound by what a workgroup can keep in flight.
template <int MB>
__global__ void __launch_bounds__(256, 1) wgrad_s2_kernel(Wg2Params P) {
    extern __shared__ __attribute__((aligned(16))) char lds[];
    constexpr int DY_BYTES = 2 * MB * DY_SLAB;
    constexpr int NDY = TH * TW * 4 * MB / 256;   // 16-byte dy pieces per thread (2 MB)
    const unsigned x_lds = (unsigned)(size_t)lds;                          // ring of XSTAGES x patches (LDS byte addresses)
    const unsigned dy_lds = x_lds + XSTAGES * X_BYTES;                     // ring of two dy patches, slot = od % 2

    const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
    const int wave_u = __builtin_amdgcn_readfirstlane(wave);
    const int coh = wave >> 1, cih = wave & 1;
    const int pair = blockIdx.y, slot = blockIdx.x;
    const int cot = pair / P.CiT, cit = pair % P.CiT;
    long long u0 = P.units * slot / P.slots, u1 = P.units * (slot + 1) / P.slots;

    // transposing reads: lane (g, s) supplies voxel 4 g + s / 4 (and + 16), channels 4 (s % 4) .. + 3 of its 16-channel half
    const int g = lane >> 4, s = lane & 15;
    const int lane_off = (4 * g + (s >> 2)) * 32 + (s & 3) * 8;                    // dy: 32 bytes per voxel and slab
    const int x_lane_off = (4 * g + (s >> 2)) * XVB + cih * 32 + (s & 3) * 8;      // x: 64 bytes per voxel

    f32x4 acc[MB][3][3][3];
#pragma unroll
    for (int m = 0; m < MB; ++m)
#pragma unroll
        for (int a = 0; a < 3; ++a)
#pragma unroll
            for (int b = 0; b < 3; ++b)
#pragma unroll
                for (int c = 0; c < 3; ++c) acc[m][a][b][c] = f32x4{0.f, 0.f, 0.f, 0.f};

    const long long x_plane = (long long)P.H * P.W * P.Cin;
    const long long dy_plane = (long long)P.Ho * P.Wo * P.Cout;

    while (u0 < u1) {
        long long column = u0 / P.D;
        const int id_start = (int)(u0 - column * P.D);
        const long long left = u1 - u0;
        const int id_end = id_start + (int)(left < (long long)(P.D - id_start) ? left : (long long)(P.D - id_start));
        u0 += id_end - id_start;
        const int wt = (int)(column % P.WT); column /= P.WT;
        const int ht = (int)(column % P.HT);
        const int n = (int)(column / P.HT);
        const int h0 = ht * TH, w0 = wt * TW;  // dy coordinates

        // Staging plans; byte offsets from the plane base, OOB (reads as zero) outside the patch or the volume.
        // x: load i of this wave is instruction 4 i + wave; lane l moves the 16-byte piece l % 4 of the voxel at staged
        // position 16 (4 i + wave) + l / 4 (row-major over 9 rows x (33 even + 33 odd columns)).
        // dy: instruction 4 i + wave fills 1 KB of the [16-cout slab][voxel][32 B] patch: slab (4 i + wave) / 4,
        // voxels 32 ((4 i + wave) % 4) + l / 2, couts 8 (l % 2) .. + 7 of the slab.
        int gx[NX], gdy[NDY];
#pragma unroll
        for (int i = 0; i < NX; ++i) {
            const int pos = 16 * (4 * i + wave) + (lane >> 2), c = lane & 3;
            const int row = (pos * 993) >> 16, rem = pos - row * XPITCH;  // pos / 66 for pos < 700
            const int par = rem >= XHALF ? 1 : 0, col = 2 * (rem - par * XHALF) + par;
            const int gh = 2 * h0 - P.pH + row, gw = 2 * w0 - P.pW + col;
            const bool ok = pos < XPOS && col < XC && gh >= 0 && gh < P.H && gw >= 0 && gw < P.W;
            gx[i] = ok ? ((gh * P.W + gw) * P.Cin + cit * 32 + c * 8) * 2 : (int)OOB;
        }
#pragma unroll
        for (int i = 0; i < NDY; ++i) {
            const int k = 4 * i + wave, slab = k >> 2, v = 32 * (k & 3) + (lane >> 1);
            const int gh = h0 + (v >> 5), gw = w0 + (v & 31);
            const bool ok = gh < P.Ho && gw < P.Wo;
            gdy[i] = ok ? ((gh * P.Wo + gw) * P.Cout + cot * 32 * MB + slab * 16 + (lane & 1) * 8) * 2 : (int)OOB;
        }
        const uint16_t* xn = P.x + (long long)n * P.D * x_plane;
        const uint16_t* dyn = P.dy + (long long)n * P.Do * dy_plane;

        // x plane id + 2 is requested during step id into the stage that step id - 1 read (every wave has passed the
        // barrier behind that step).  dy plane m + 1 is requested at the start of the odd step 2 m + 1 into the ring
        // slot that only even steps read, ahead of that step's x requests.  A plane outside the volume (for x also:
        // past the end of the segment) gets a buffer of zero records: its pieces read as zero and nothing is fetched.
        // At the end of every step all requests but this step's NX x pieces must have arrived.  One barrier per step.
        auto load_x_plane_piece = [&](int i, int stage, u32x4 rsrc) {
            dma16(rsrc, x_lds + stage * X_BYTES + (4 * i + wave_u) * 1024, gx[i]);
        };
        auto x_rsrc = [&](int id) {
            const bool in = id >= 0 && id < id_end;
            return make_rsrc(xn + (long long)(in ? id : 0) * x_plane, in ? (unsigned)(x_plane * 2) : 0u);
        };
        auto load_dy_plane = [&](int od) {
            const bool in = od >= 0 && od < P.Do;
            const u32x4 r = make_rsrc(dyn + (long long)(in ? od : 0) * dy_plane, in ? (unsigned)(dy_plane * 2) : 0u);
#pragma unroll
            for (int i = 0; i < NDY; ++i) dma16(r, dy_lds + (od & 1) * DY_BYTES + (4 * i + wave_u) * 1024, gdy[i]);
        };
        // dy planes an x plane needs: tp = id + pD; even tp: od = tp/2 (kd 0) and tp/2 - 1 (kd 2); odd: (tp-1)/2 (kd 1)
        auto floor_half = [](int v) { return (v - (v & 1)) / 2; };  // floor(v / 2) for negative v too

        {   // the first x plane and the dy planes of the first step, then the second x plane (which may still fly)
            const u32x4 r0 = x_rsrc(id_start), r1 = x_rsrc(id_start + 1);
#pragma unroll
            for (int i = 0; i < NX; ++i) load_x_plane_piece(i, 0, r0);
            const int m = floor_half(id_start + P.pD);
            load_dy_plane(m - 1);
            load_dy_plane(m);
#pragma unroll
            for (int i = 0; i < NX; ++i) load_x_plane_piece(i, 1, r1);
        }
        WG2_WAIT_AND_BARRIER(NX);

        int sq = 0;
        for (int id = id_start; id < id_end; ++id, ++sq) {
            const int tp = id + P.pD;
            const bool even = (tp & 1) == 0;
            const int m = floor_half(tp);
            const char* x_lane = lds + (sq % XSTAGES) * X_BYTES + x_lane_off;
            const int fill = (sq + 2) % XSTAGES;
            const char* dy_base = lds + XSTAGES * X_BYTES + coh * MB * DY_SLAB + lane_off;
            const char* const dy_lane[2] = {dy_base + (m & 1) * DY_BYTES, dy_base + ((m - 1) & 1) * DY_BYTES};
            const u32x4 rx = x_rsrc(id + 2);
            // hook schedule: the ten x loads in rows 0..4 (two each)
            if (even) {
                plane_step<true, MB>(acc, x_lane, dy_lane, [&](int r) {
#pragma unroll
                    for (int j = 0; j < 2; ++j)
                        if (2 * r + j < NX) load_x_plane_piece(2 * r + j, fill, rx);
                });
            } else {
                load_dy_plane(m + 1);
                plane_step<false, MB>(acc, x_lane, dy_lane, [&](int r) {
#pragma unroll
                    for (int j = 0; j < 2; ++j)
                        if (2 * r + j < NX) load_x_plane_piece(2 * r + j, fill, rx);
                });
            }
            WG2_WAIT_AND_BARRIER(NX);
        }
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // the zero-record requests of the last steps

    float* out = P.part + (long long)slot * ((long long)P.Cout * 27 * P.Cin);
#pragma unroll
    for (int b = 0; b < MB; ++b)
#pragma unroll
        for (int kd = 0; kd < 3; ++kd)
#pragma unroll
            for (int kh = 0; kh < 3; ++kh)
#pragma unroll
                for (int kw = 0; kw < 3; ++kw) {
                    const int tap = (kd * 3 + kh) * 3 + kw;
#pragma unroll
                    for (int v = 0; v < 4; ++v) {
                        const int co = (cot * 2 + coh) * 16 * MB + b * 16 + 4 * (lane >> 4) + v;
                        const int ci = cit * 32 + cih * 16 + (lane & 15);
                        out[((long long)co * 27 + tap) * P.Cin + ci] = acc[b][kd][kh][kw][v];
                    }
                }
}

}  // namespace

bool wgrad_s2_supported(const Geom& g) {
    if (g.dtype != MI3D_BF16 || g.kD != 3 || g.kH != 3 || g.kW != 3) return false;
    if (g.sD != 2 || g.sH != 2 || g.sW != 2) return false;
    if (g.pD > 1 || g.pH > 1 || g.pW > 1) return false;
    // a staged x plane is addressed through a buffer resource with 32-bit byte offsets; 2^31 marks padding
    if ((long long)g.H * g.W * g.Cin * 2 >= (1ll << 31) || (long long)g.Ho * g.Wo * g.Cout * 2 >= (1ll << 31)) return false;
    return g.Cin % 32 == 0 && g.Cout % 32 == 0;
}

static int wgrad_s2_mb(const Geom& g) { return g.Cout % 64 == 0 ? 2 : 1; }

static int wgrad_s2_slots(const Geom& g) {
    long long pairs = (long long)(g.Cin / 32) * (g.Cout / (32 * wgrad_s2_mb(g)));
    long long units = (long long)g.N * ((g.Ho + TH - 1) / TH) * ((g.Wo + TW - 1) / TW) * g.D;
    long long slots = (256 + pairs - 1) / pairs;
    if (slots > units) slots = units;
    if (slots < 1) slots = 1;
    return (int)slots;
}

size_t wgrad_s2_workspace_bytes(const Geom& g) {
    if (!wgrad_s2_supported(g)) return 0;
    return (size_t)wgrad_s2_slots(g) * g.w_elems() * sizeof(float);
}

int wgrad_s2(const Geom& g, const void* x, const void* dy, float* dw, void* ws, size_t ws_bytes, hipStream_t s) {
    if (ws_bytes < wgrad_s2_workspace_bytes(g)) return MI3D_ERR_WORKSPACE;
    Wg2Params P;
    P.x = (const uint16_t*)x; P.dy = (const uint16_t*)dy; P.part = (float*)ws;
    P.N = g.N; P.D = g.D; P.H = g.H; P.W = g.W; P.Cin = g.Cin; P.Cout = g.Cout;
    P.Do = g.Do; P.Ho = g.Ho; P.Wo = g.Wo; P.pD = g.pD; P.pH = g.pH; P.pW = g.pW;
    P.HT = (g.Ho + TH - 1) / TH;
    P.WT = (g.Wo + TW - 1) / TW;
    P.CiT = g.Cin / 32;
    const int mb = wgrad_s2_mb(g);
    P.CoT = g.Cout / (32 * mb);
    P.units = (long long)g.N * P.HT * P.WT * g.D;
    P.slots = wgrad_s2_slots(g);
    const int pairs = P.CiT * P.CoT;
    if (pairs > 65535) return MI3D_ERR_UNSUPPORTED;
    const size_t lds = XSTAGES * X_BYTES + 2 * (size_t)(2 * mb * DY_SLAB);
    static std::atomic<bool> attr_set{false};   // set once per process; a second thread racing here repeats an idempotent call
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute((const void*)wgrad_s2_kernel<1>, hipFuncAttributeMaxDynamicSharedMemorySize, XSTAGES * X_BYTES + 4 * DY_SLAB);
        if (e == hipSuccess) e = hipFuncSetAttribute((const void*)wgrad_s2_kernel<2>, hipFuncAttributeMaxDynamicSharedMemorySize, XSTAGES * X_BYTES + 8 * DY_SLAB);
        if (e != hipSuccess) { note_hip_error(e); return MI3D_ERR_HIP; }
        attr_set = true;
    }
    if (mb == 2) wgrad_s2_kernel<2><<<dim3((unsigned)P.slots, (unsigned)pairs), 256, lds, s>>>(P);
    else wgrad_s2_kernel<1><<<dim3((unsigned)P.slots, (unsigned)pairs), 256, lds, s>>>(P);
    int st = check_launch();
    if (st) return st;
    long long n = g.w_elems();
    return reduce_partials((const float*)ws, dw, n, P.slots, s);
}

}  // namespace mi3d
