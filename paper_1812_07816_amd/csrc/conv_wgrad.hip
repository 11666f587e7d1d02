// Weight gradient of 3x3x3 / stride 1 layers on bf16 MFMA
// (v_mfma_f32_16x16x32_bf16), fp32 accumulation and fp32 output:
//   dw[co,t,ci] = sum_{n,o} dy[n,o,co] * x[n, o - p + t, ci]
// the pass that needs the saved input feature map of the layer (Section 3.1).
//
// The contraction runs over voxels, which are strided by the channel count in
// NDHWC, so both MFMA operands need a transposing read: tiles are staged in
// LDS as [16-channel slab][row][voxel] and fetched with ds_read_b64_tr_b16,
// which hands each lane 4 consecutive voxels of one channel.
//
// Work decomposition
//   pair    = (32-wide cout tile, 32-wide cin tile); a workgroup serves one pair
//   column  = (n, 16-row x 32-col patch of the dy plane)
//   unit    = (column, x plane id); contiguous unit ranges per workgroup.
//   A step stages one x plane patch with halo (18 x 34 voxels) and keeps a ring
//   of the three dy plane patches od = id + pD - kd.  Each of the 4 waves owns
//   a 16x16 (co, ci) quadrant for all 27 taps (27 accumulators of 4 registers)
//   and walks the 18 x rows: an x fragment (one per kw) meets the 3x3 window
//   of dy fragments (kd, kh) held in registers, so one LDS fragment feeds 9
//   MFMAs.  Partial sums go to a per-workgroup slot of the workspace and are
//   added in slot order by a second kernel, which makes the result
//   bit-reproducible.
#include "mi3d_internal.h"

// The file is compiled twice: as it is (16-row patches, namespace th16) and from conv_wgrad12.hip with 12-row patches
// (namespace th12) for planes whose height 16-row patches cover badly (24 and 12 rows: a quarter of the MFMA work
// would fall on rows outside the tensor).  The entry points at the end of the 16-row build choose between the two.
#ifndef WG_TH
#define WG_TH 16
#define WG_NS th16
#endif

namespace mi3d {
namespace WG_NS {
namespace {

typedef __attribute__((__vector_size__(4 * sizeof(short)))) short s16x4;
typedef __attribute__((__vector_size__(8 * sizeof(short)))) short s16x8;
typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float f32x4;

constexpr int TH = WG_TH, TW = 32;
// PAIRED (12-row build): where the last column of patches has at most 16 columns inside the tensor (W = 48: 32 + 16),
// a workgroup takes that column for two patch rows at once: voxels 0..15 of a staged dy row are the 16 columns of
// patch row 2 i, voxels 16..31 the same columns of patch row 2 i + 1, so no MFMA k-step is spent outside the tensor.
// The two x patches (18 columns each with halo) sit side by side in the staged rows.
constexpr bool PAIRED = TH == 12;
constexpr int HALF = TW / 2 + 2;                 // staged columns of one half of a paired x patch
constexpr int XR = TH + 2, XC = PAIRED ? 2 * HALF : TW + 2;   // x patch with halo
constexpr int X_SLAB = XR * XC * 32;             // bytes of one 16-channel slab of the x patch
constexpr int X_BYTES = 2 * X_SLAB;
constexpr int DY_SLAB = TH * TW * 32;
constexpr int DY_BYTES = 2 * DY_SLAB;
constexpr int NX = (XR * XC * 4 + 255) / 256;    // 16-byte pieces per thread: x patch (10)
constexpr int NDY = TH * TW * 4 / 256;           // dy patch (8)
constexpr int XPIECES = XR * XC * 4;
static_assert(NX + NDY <= XR && NDY * 256 == TH * TW * 4, "one global load per x row covers both patches");

struct WgParams {
    const uint16_t* x;
    const uint16_t* dy;
    float* part;            // [slots][Cout][27][Cin]
    int N, D, H, W, Cin, Cout, Do, Ho, Wo, pD, pH, pW;
    int HT, WT, CiT, CoT;
    int WTF, HTP;           // columns of patches taken one patch at a time, paired patch rows of the last column (else 0)
    long long units;        // per pair: N*HT*WT*D
    int slots;              // workgroups per pair
    // x given as two halves along the channels (virtual concatenation): cin tiles >= xsplit come from x2; xpitch is
    // the channels per voxel of x in memory (Cin when not split; then xsplit lies beyond the last tile)
    const uint16_t* x2;
    int xpitch, xsplit;
};

__device__ __forceinline__ bf16x8 tr_frag(const char* p) {
    typedef __attribute__((address_space(3))) s16x4* lptr;
    s16x4 a = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lptr)(p));
    s16x4 b = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lptr)(p + 16 * 32));  // voxels +16
    s16x8 c = __builtin_shufflevector(a, b, 0, 1, 2, 3, 4, 5, 6, 7);
    return __builtin_bit_cast(bf16x8, c);
}

// the same with the second sixteen voxels at an address of their own (paired x patches)
__device__ __forceinline__ bf16x8 tr_frag2(const char* p, const char* p2) {
    typedef __attribute__((address_space(3))) s16x4* lptr;
    s16x4 a = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lptr)(p));
    s16x4 b = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lptr)(p2));
    s16x8 c = __builtin_shufflevector(a, b, 0, 1, 2, 3, 4, 5, 6, 7);
    return __builtin_bit_cast(bf16x8, c);
}

__device__ __forceinline__ f32x4 mfma16(bf16x8 a, bf16x8 b, f32x4 c) {
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, c, 0, 0, 0);
}

#define WG_FENCE() __builtin_amdgcn_sched_barrier(0)

// x row R of the patch against the dy rows R - kh.  dyw[kd][slot] is the
// register window of dy fragments, slot = dy row mod 4; xf holds the three kw
// shifts of the current row, xn receives those of the next row.
template <int R, class Hook>
__device__ __forceinline__ void row_step(f32x4 (&acc)[3][3][3], bf16x8 (&dyw)[3][4], bf16x8 (&xf)[3], bf16x8 (&xn)[3],
                                         const char* x_lane, const char* x_lane2, const char* const (&dy_lane)[3], Hook&& hook) {
    // prefetch for row R + 1: its dy fragments (one per kd) and x fragments (one per kw)
    if (R + 1 < TH) {
#pragma unroll
        for (int kd = 0; kd < 3; ++kd) dyw[kd][(R + 1) % 4] = tr_frag(dy_lane[kd] + (R + 1) * TW * 32);
    }
    if (R + 1 < XR) {
#pragma unroll
        for (int kw = 0; kw < 3; ++kw) xn[kw] = tr_frag2(x_lane + ((R + 1) * XC + kw) * 32, x_lane2 + ((R + 1) * XC + kw) * 32);
    }
#pragma unroll
    for (int kh = 0; kh < 3; ++kh) {
        constexpr int dummy = 0; (void)dummy;
        const int dr = R - kh;  // dy row fed by this x row through tap kh
        if (dr < 0 || dr >= TH) continue;
#pragma unroll
        for (int kd = 0; kd < 3; ++kd)
#pragma unroll
            for (int kw = 0; kw < 3; ++kw) acc[kd][kh][kw] = mfma16(dyw[kd][dr % 4], xf[kw], acc[kd][kh][kw]);
    }
    hook(R);
    WG_FENCE();
}

// rows R, R + 1, ... of the x patch; xf holds the fragments of row R, the other set receives those of row R + 1
template <int R, class Hook>
__device__ __forceinline__ void rows_from(f32x4 (&acc)[3][3][3], bf16x8 (&dyw)[3][4], bf16x8 (&xf)[3], bf16x8 (&xn)[3],
                                          const char* x_lane, const char* x_lane2, const char* const (&dy_lane)[3], Hook&& hook) {
    if constexpr (R < XR) {
        row_step<R>(acc, dyw, xf, xn, x_lane, x_lane2, dy_lane, hook);
        rows_from<R + 1>(acc, dyw, xn, xf, x_lane, x_lane2, dy_lane, hook);
    }
}

template <class Hook>
__device__ __forceinline__ void plane_step(f32x4 (&acc)[3][3][3], const char* x_lane, const char* x_lane2, const char* const (&dy_lane)[3], Hook&& hook) {
    bf16x8 dyw[3][4], xa[3], xb[3];
#pragma unroll
    for (int kd = 0; kd < 3; ++kd) dyw[kd][0] = tr_frag(dy_lane[kd]);
#pragma unroll
    for (int kw = 0; kw < 3; ++kw) xa[kw] = tr_frag2(x_lane + kw * 32, x_lane2 + kw * 32);
    rows_from<0>(acc, dyw, xa, xb, x_lane, x_lane2, dy_lane, hook);
}

__device__ __forceinline__ int mod3(int v) { return ((v % 3) + 3) % 3; }

__global__ void __launch_bounds__(256, 1) wgrad_kernel(WgParams P) {
    extern __shared__ __attribute__((aligned(16))) char lds[];
    char* x_lds = lds;                 // one x patch
    char* dy_lds = lds + X_BYTES;      // ring of three dy patches

    const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
    const int coh = wave >> 1, cih = wave & 1;   // 16x16 quadrant of the 32x32 (co, ci) tile
    const int pair = blockIdx.y, slot = blockIdx.x;
    const int cot = pair / P.CiT, cit = pair % P.CiT;
    long long u0 = P.units * slot / P.slots, u1 = P.units * (slot + 1) / P.slots;

    // per-lane part of the transposing reads: lane group g covers voxels 4g..4g+3
    // (and +16 in the second read), lane s within the group supplies row s/4, channels 4(s%4)..
    const int g = lane >> 4, s = lane & 15;
    const int lane_off = (4 * g + (s >> 2)) * 32 + (s & 3) * 8;
    const char* x_lane = x_lds + cih * X_SLAB + lane_off;

    f32x4 acc[3][3][3];
#pragma unroll
    for (int a = 0; a < 3; ++a)
#pragma unroll
        for (int b = 0; b < 3; ++b)
#pragma unroll
            for (int c = 0; c < 3; ++c) acc[a][b][c] = f32x4{0.f, 0.f, 0.f, 0.f};

    const long long x_plane = (long long)P.H * P.W * P.xpitch;
    const bool x_high = cit >= P.xsplit;
    const int cit_local = x_high ? cit - P.xsplit : cit;
    const long long dy_plane = (long long)P.Ho * P.Wo * P.Cout;

    while (u0 < u1) {
        long long column = u0 / P.D;
        const int id_start = (int)(u0 - column * P.D);
        const long long left = u1 - u0;
        const int id_end = id_start + (int)(left < (long long)(P.D - id_start) ? left : (long long)(P.D - id_start));
        u0 += id_end - id_start;
        const int tpp = P.HT * P.WTF + P.HTP;                  // patches of a plane
        const int tsel = (int)(column % tpp);
        const int n = (int)(column / tpp);
        const bool paired = PAIRED && tsel >= P.HT * P.WTF;    // (uniform)
        const int wtf1 = P.WTF > 0 ? P.WTF : 1;                // (no unpaired column: every patch is paired)
        const int wt = paired ? P.WTF : tsel % wtf1;
        const int ht = paired ? 2 * (tsel - P.HT * P.WTF) : tsel / wtf1;
        const int h0 = ht * TH, w0 = wt * TW;
        // the second sixteen voxels of an x fragment: the same staged row, or the second patch's part of it
        const char* x_lane2 = x_lane + (16 + (paired ? HALF - 16 : 0)) * 32;

        // load plans: x piece q = t + 256 i is channels 8c..8c+7 of patch voxel q / 4
        int gx[NX], gdy[NDY];
        unsigned vx = 0, vdy = 0;
#pragma unroll
        for (int i = 0; i < NX; ++i) {
            int q = t + 256 * i, v = q >> 2, c = q & 3;
            int row = v / XC, col = v - row * XC;
            const bool second = paired && col >= HALF;   // the patch one patch row further down
            int gh = h0 + (second ? TH : 0) - P.pH + row, gw = w0 - P.pW + (second ? col - HALF : col);
            bool ok = q < XPIECES && col < (paired ? XC : TW + 2) && gh >= 0 && gh < P.H && gw >= 0 && gw < P.W;
            gx[i] = ok ? (gh * P.W + gw) * P.xpitch + cit_local * 32 + c * 8 : 0;
            vx |= (ok ? 1u : 0u) << i;
        }
#pragma unroll
        for (int i = 0; i < NDY; ++i) {
            int q = t + 256 * i, v = q >> 2, c = q & 3;
            int row = v >> 5, col = v & 31;
            const bool second = paired && col >= 16;
            int gh = h0 + (second ? TH : 0) + row, gw = w0 + (second ? col - 16 : col);
            bool ok = gh < P.Ho && gw < P.Wo && !(paired && !second && col >= 16);
            gdy[i] = ok ? (gh * P.Wo + gw) * P.Cout + cot * 32 + c * 8 : 0;
            vdy |= (ok ? 1u : 0u) << i;
        }
        const uint16_t* xn = (x_high ? P.x2 : P.x) + (long long)n * P.D * x_plane;
        const uint16_t* dyn = P.dy + (long long)n * P.Do * dy_plane;

        uint4 px[NX], pdy[NDY];
        unsigned mx = 0, mdy = 0;
        const uint16_t *bx = xn, *bdy = dyn;
        auto begin_x = [&](int id) {
            const bool in = id >= 0 && id < P.D;
            bx = xn + (long long)(in ? id : 0) * x_plane;
            mx = in ? vx : 0u;
        };
        auto begin_dy = [&](int od) {
            const bool in = od >= 0 && od < P.Do;
            bdy = dyn + (long long)(in ? od : 0) * dy_plane;
            mdy = in ? vdy : 0u;
        };
        auto write_x = [&]() {
#pragma unroll
            for (int i = 0; i < NX; ++i) {
                int q = t + 256 * i, v = q >> 2, c = q & 3;
                int row = v / XC, col = v - row * XC;
                const bool ok = (mx >> i) & 1;
                uint4 w;
                w.x = ok ? px[i].x : 0u; w.y = ok ? px[i].y : 0u; w.z = ok ? px[i].z : 0u; w.w = ok ? px[i].w : 0u;
                if (q < XPIECES) *(uint4*)(x_lds + (c >> 1) * X_SLAB + (row * XC + col) * 32 + (c & 1) * 16) = w;
            }
        };
        auto write_dy = [&](int ring) {
            char* dst = dy_lds + ring * DY_BYTES;
#pragma unroll
            for (int i = 0; i < NDY; ++i) {
                int q = t + 256 * i, v = q >> 2, c = q & 3;
                const bool ok = (mdy >> i) & 1;
                uint4 w;
                w.x = ok ? pdy[i].x : 0u; w.y = ok ? pdy[i].y : 0u; w.z = ok ? pdy[i].z : 0u; w.w = ok ? pdy[i].w : 0u;
                *(uint4*)(dst + (c >> 1) * DY_SLAB + v * 32 + (c & 1) * 16) = w;
            }
        };

        // prologue: x plane id_start and the dy planes of its three kd taps
        __syncthreads();  // previous segment's readers are done with the LDS
        begin_x(id_start);
#pragma unroll
        for (int i = 0; i < NX; ++i) px[i] = *(const uint4*)(bx + gx[i]);
        write_x();
        for (int kd = 0; kd < 3; ++kd) {
            const int od = id_start + P.pD - kd;
            begin_dy(od);
#pragma unroll
            for (int i = 0; i < NDY; ++i) pdy[i] = *(const uint4*)(bdy + gdy[i]);
            write_dy(mod3(od));
        }
        __syncthreads();

        for (int id = id_start; id < id_end; ++id) {
            const bool more = id + 1 < id_end;
            begin_x(id + 1);
            begin_dy(id + 1 + P.pD);  // the plane that enters the ring for the next step
            const char* dyl[3];
#pragma unroll
            for (int kd = 0; kd < 3; ++kd)
                dyl[kd] = dy_lds + mod3(id + P.pD - kd) * DY_BYTES + coh * DY_SLAB + lane_off;
            const char* const dy_lane[3] = {dyl[0], dyl[1], dyl[2]};
            // one global load per x row: the first NX rows fetch the next x patch, the other NDY the next dy patch.
            // The loads and the LDS writes below are unconditional (the step after the last one of a segment
            // fetches a valid plane that is never used): with a condition the compiler cannot pair each
            // load with its consumer and waits for all outstanding loads before every new one.
            (void)more;
            plane_step(acc, x_lane, x_lane2, dy_lane, [&](int r) {
                if (r < NX) px[r] = *(const uint4*)(bx + gx[r]);
                else if (r - NX < NDY) pdy[r - NX] = *(const uint4*)(bdy + gdy[r - NX]);
            });
            __syncthreads();  // everyone is done reading the x patch and the oldest dy patch
            write_x();
            write_dy(mod3(id + 1 + P.pD));
            __syncthreads();
        }
    }

    // partial sums of this workgroup: acc register v of lane l is
    // (co = 4 (l / 16) + v, ci = l % 16) of the quadrant
    float* out = P.part + (long long)slot * ((long long)P.Cout * 27 * P.Cin);
#pragma unroll
    for (int kd = 0; kd < 3; ++kd)
#pragma unroll
        for (int kh = 0; kh < 3; ++kh)
#pragma unroll
            for (int kw = 0; kw < 3; ++kw) {
                const int tap = (kd * 3 + kh) * 3 + kw;
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    const int co = cot * 32 + coh * 16 + 4 * (lane >> 4) + v;
                    const int ci = cit * 32 + cih * 16 + (lane & 15);
                    out[((long long)co * 27 + tap) * P.Cin + ci] = acc[kd][kh][kw][v];
                }
            }
}

}  // namespace

bool supported(const Geom& g) {
    if (g.dtype != MI3D_BF16 || g.kD != 3 || g.kH != 3 || g.kW != 3) return false;
    if (g.sD != 1 || g.sH != 1 || g.sW != 1) return false;
    if (g.pD > 2 || g.pH > 2 || g.pW > 2) return false;
    if (!g.planes_fit_32bit()) return false;
    return g.Cin % 32 == 0 && g.Cout % 32 == 0;
}

// Patches of a dy plane of Ho x Wo: wtf columns of patches are taken one patch at a time; where the last column has
// at most 16 columns inside the tensor and there are at least two patch rows, it is taken two patch rows at a time
// (htp pairs; 12-row build only).
static int plane_tiles(int Ho, int Wo, int* wtf, int* htp) {
    const int HT = (Ho + TH - 1) / TH, WT = (Wo + TW - 1) / TW, tail = Wo - (WT - 1) * TW;
    const bool pair = PAIRED && tail <= TW / 2 && HT >= 2;
    *wtf = pair ? WT - 1 : WT;
    *htp = pair ? (HT + 1) / 2 : 0;
    return HT * *wtf + *htp;
}

static int wgrad_slots(const Geom& g) {
    long long pairs = (long long)(g.Cin / 32) * (g.Cout / 32);
    int wtf, htp;
    long long units = (long long)g.N * plane_tiles(g.Ho, g.Wo, &wtf, &htp) * g.D;
    long long slots = (256 + pairs - 1) / pairs;   // about one workgroup per CU in total
    if (slots > units) slots = units;
    if (slots < 1) slots = 1;
    return (int)slots;
}

size_t workspace_bytes(const Geom& g) {
    if (!supported(g)) return 0;
    return (size_t)wgrad_slots(g) * g.w_elems() * sizeof(float);
}

int run(const Geom& g, const void* x, const void* dy, float* dw, void* ws, size_t ws_bytes, hipStream_t s) {
    if (ws_bytes < workspace_bytes(g)) return MI3D_ERR_WORKSPACE;
    WgParams P;
    P.x = (const uint16_t*)x;
    P.dy = (const uint16_t*)dy;
    P.part = (float*)ws;
    P.N = g.N; P.D = g.D; P.H = g.H; P.W = g.W; P.Cin = g.Cin; P.Cout = g.Cout;
    P.Do = g.Do; P.Ho = g.Ho; P.Wo = g.Wo; P.pD = g.pD; P.pH = g.pH; P.pW = g.pW;
    P.HT = (g.Ho + TH - 1) / TH;
    P.WT = (g.Wo + TW - 1) / TW;
    P.CiT = g.Cin / 32;
    P.CoT = g.Cout / 32;
    P.units = (long long)g.N * plane_tiles(g.Ho, g.Wo, &P.WTF, &P.HTP) * g.D;
    P.slots = wgrad_slots(g);
    P.x2 = P.x; P.xpitch = g.Cin; P.xsplit = P.CiT;
    if (g.hi) {
        if (g.Cin % 64) return MI3D_ERR_UNSUPPORTED;
        P.x2 = (const uint16_t*)g.hi; P.xpitch = g.Cin / 2; P.xsplit = P.CiT / 2;
    }
    const int pairs = P.CiT * P.CoT;
    if (pairs > 65535) return MI3D_ERR_UNSUPPORTED;
    size_t lds = X_BYTES + 3 * DY_BYTES;
    static std::atomic<bool> attr_set{false};   // set once per process; a second thread racing here repeats an idempotent call
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute((const void*)wgrad_kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) { note_hip_error(e); return MI3D_ERR_HIP; }
        attr_set = true;
    }
    wgrad_kernel<<<dim3((unsigned)P.slots, (unsigned)pairs), 256, lds, s>>>(P);
    int st = check_launch();
    if (st) return st;
    long long n = g.w_elems();
    return reduce_partials((const float*)ws, dw, n, P.slots, s);
}

}  // namespace WG_NS

#if WG_TH == 16
namespace th12 {
size_t workspace_bytes(const Geom& g);
int run(const Geom& g, const void* x, const void* dy, float* dw, void* ws, size_t ws_bytes, hipStream_t s);
}  // namespace th12

// 12-row patches where they cover the dy plane with fewer rows than 16-row patches do (heights 12, 24, 36, ...)
// and on a tie where the last column of patches can be paired (widths 48, 16, ...)
static bool wgrad_rows12(const Geom& g) {
    const int r16 = (g.Ho + 15) / 16 * 16, r12 = (g.Ho + 11) / 12 * 12;
    if (r12 != r16) return r12 < r16;
    const int tail = g.Wo - (g.Wo - 1) / 32 * 32;
    return tail <= 16 && r12 >= 24;
}

bool wgrad_mfma_supported(const Geom& g) { return th16::supported(g); }
size_t wgrad_mfma_workspace_bytes(const Geom& g) { return wgrad_rows12(g) ? th12::workspace_bytes(g) : th16::workspace_bytes(g); }
int wgrad_mfma(const Geom& g, const void* x, const void* dy, float* dw, void* ws, size_t ws_bytes, hipStream_t s) {
    return wgrad_rows12(g) ? th12::run(g, x, dy, dw, ws, ws_bytes, s) : th16::run(g, x, dy, dw, ws, ws_bytes, s);
}
#endif

}  // namespace mi3d
