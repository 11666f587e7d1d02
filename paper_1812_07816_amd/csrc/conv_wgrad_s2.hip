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
// 2 j + kw of a fragment are contiguous in LDS.
#include "mi3d_internal.h"

namespace mi3d {
namespace {

typedef __attribute__((__vector_size__(4 * sizeof(short)))) short s16x4;
typedef __attribute__((__vector_size__(8 * sizeof(short)))) short s16x8;
typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float f32x4;

constexpr int TH = 4, TW = 32;
constexpr int XR = 2 * TH + 1, XC = 2 * TW + 1;  // 9 x 65
constexpr int XHALF = 33, XPITCH = 2 * XHALF;    // even columns, then odd columns
constexpr int X_SLAB = XR * XPITCH * 32;
constexpr int X_BYTES = 2 * X_SLAB;
constexpr int DY_SLAB = TH * TW * 32;
constexpr int DY_BYTES = 2 * DY_SLAB;
constexpr int XPIECES = XR * XC * 4;
constexpr int NX = (XPIECES + 255) / 256;        // 10
constexpr int NDY = TH * TW * 4 / 256;           // 2

struct Wg2Params {
    const uint16_t* x;
    const uint16_t* dy;
    float* part;
    int N, D, H, W, Cin, Cout, Do, Ho, Wo, pD, pH, pW;
    int HT, WT, CiT, CoT;
    long long units;  // per pair: N*HT*WT*D
    int slots;
};

__device__ __forceinline__ bf16x8 tr_frag(const char* p) {
    typedef __attribute__((address_space(3))) s16x4* lptr;
    s16x4 a = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lptr)(p));
    s16x4 b = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lptr)(p + 16 * 32));
    s16x8 c = __builtin_shufflevector(a, b, 0, 1, 2, 3, 4, 5, 6, 7);
    return __builtin_bit_cast(bf16x8, c);
}

__device__ __forceinline__ f32x4 mfma16(bf16x8 a, bf16x8 b, f32x4 c) {
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, c, 0, 0, 0);
}

// One staged x plane.  EVEN: id + pD even, taps kd 0 (dy plane in dy_lane[0]) and kd 2 (dy_lane[1]);
// otherwise tap kd 1 (dy_lane[0]).  x row R meets dy row dr through kh = R - 2 dr.
template <bool EVEN, class Hook>
__device__ __forceinline__ void plane_step(f32x4 (&acc)[3][3][3], const char* x_lane, const char* const (&dy_lane)[2], Hook&& hook) {
    constexpr int NKD = EVEN ? 2 : 1;
    bf16x8 dyw[NKD][3];  // window over dy rows, slot = dr % 3
#pragma unroll
    for (int k = 0; k < NKD; ++k) dyw[k][0] = tr_frag(dy_lane[k]);
    // x fragments are read three rows ahead of their use (ring of four); left to the compiler every row is
    // read -> wait -> MFMAs, and with 3 to 12 MFMAs per row two rows do not cover the LDS latency
    constexpr int AH = 3;
    bf16x8 xf[AH + 1][3];
    auto load_xrow = [&](int R) {
#pragma unroll
        for (int kw = 0; kw < 3; ++kw) xf[R % (AH + 1)][kw] = tr_frag(x_lane + (R * XPITCH + (kw & 1) * XHALF + (kw >> 1)) * 32);
    };
#pragma unroll
    for (int R = 0; R < AH; ++R) load_xrow(R);
#pragma unroll
    for (int R = 0; R < XR; ++R) {
        if (R + AH < XR) load_xrow(R + AH);
        if ((R & 1) == 0 && R / 2 + 1 < TH) {  // the dy row that the next even x row starts using
#pragma unroll
            for (int k = 0; k < NKD; ++k) dyw[k][(R / 2 + 1) % 3] = tr_frag(dy_lane[k] + (R / 2 + 1) * TW * 32);
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
                for (int kw = 0; kw < 3; ++kw) acc[kd][kh][kw] = mfma16(dyw[k][dr % 3], xf[R % (AH + 1)][kw], acc[kd][kh][kw]);
            }
        }
        hook(R);
        __builtin_amdgcn_sched_barrier(0);
    }
}

__global__ void __launch_bounds__(256, 1) wgrad_s2_kernel(Wg2Params P) {
    extern __shared__ __attribute__((aligned(16))) char lds[];
    char* x_lds = lds;                 // two x patches, slot = id % 2
    char* dy_lds = lds + 2 * X_BYTES;  // ring of two dy patches, slot = od % 2

    const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
    const int coh = wave >> 1, cih = wave & 1;
    const int pair = blockIdx.y, slot = blockIdx.x;
    const int cot = pair / P.CiT, cit = pair % P.CiT;
    long long u0 = P.units * slot / P.slots, u1 = P.units * (slot + 1) / P.slots;

    const int g = lane >> 4, s = lane & 15;
    const int lane_off = (4 * g + (s >> 2)) * 32 + (s & 3) * 8;
    const int x_lane_off = cih * X_SLAB + lane_off;
    // LDS offsets of the pieces this thread stages (the same for every tile)
    int lx[NX], ldy[NDY];
#pragma unroll
    for (int i = 0; i < NX; ++i) {
        const int q = t + 256 * i, v = q >> 2, c = q & 3;
        const int row = (v * 1009) >> 16, col = v - row * XC;  // v / 65
        lx[i] = (c >> 1) * X_SLAB + (row * XPITCH + (col & 1) * XHALF + (col >> 1)) * 32 + (c & 1) * 16;
    }
#pragma unroll
    for (int i = 0; i < NDY; ++i) {
        const int q = t + 256 * i, v = q >> 2, c = q & 3;
        ldy[i] = (c >> 1) * DY_SLAB + v * 32 + (c & 1) * 16;
    }

    f32x4 acc[3][3][3];
#pragma unroll
    for (int a = 0; a < 3; ++a)
#pragma unroll
        for (int b = 0; b < 3; ++b)
#pragma unroll
            for (int c = 0; c < 3; ++c) acc[a][b][c] = f32x4{0.f, 0.f, 0.f, 0.f};

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

        int gx[NX], gdy[NDY];
        unsigned vx = 0, vdy = 0;
#pragma unroll
        for (int i = 0; i < NX; ++i) {
            const int q = t + 256 * i, v = q >> 2, c = q & 3;
            const int row = (v * 1009) >> 16, col = v - row * XC;  // v / 65
            const int gh = 2 * h0 - P.pH + row, gw = 2 * w0 - P.pW + col;
            const bool ok = q < XPIECES && gh >= 0 && gh < P.H && gw >= 0 && gw < P.W;
            gx[i] = ok ? (gh * P.W + gw) * P.Cin + cit * 32 + c * 8 : 0;
            vx |= (ok ? 1u : 0u) << i;
        }
#pragma unroll
        for (int i = 0; i < NDY; ++i) {
            const int q = t + 256 * i, v = q >> 2, c = q & 3;
            const int row = v >> 5, col = v & 31;
            const int gh = h0 + row, gw = w0 + col;
            const bool ok = gh < P.Ho && gw < P.Wo;
            gdy[i] = ok ? (gh * P.Wo + gw) * P.Cout + cot * 32 + c * 8 : 0;
            vdy |= (ok ? 1u : 0u) << i;
        }
        const uint16_t* xn = P.x + (long long)n * P.D * x_plane;
        const uint16_t* dyn = P.dy + (long long)n * P.Do * dy_plane;

        // Global loads run two planes ahead of the MFMAs and the LDS writes one plane ahead, both spread
        // over the rows of the step that is being computed: during step id, piece r of x plane id + 2 is
        // requested into the register set of its parity, and piece r of plane id + 1 (requested a step
        // earlier) goes from the other set into the x buffer that step id + 1 will read.  dy plane m + 1 is
        // requested during the even step 2 m and written during the odd step 2 m + 1 into the ring slot that
        // only even steps read.  One barrier per step.  (Measured before: with the writes gathered at the
        // end of the step between two barriers they cost 40 % of the kernel's time.)  Loads and writes are
        // unconditional; planes outside the volume read plane 0 and are zeroed.
        uint4 px[2][NX], pdy[NDY];
        unsigned mx[2] = {0u, 0u}, mdy = 0;
        const uint16_t* bx[2] = {xn, xn};
        const uint16_t* bdy = dyn;
        auto begin_x = [&](int set, int id) {
            const bool in = id >= 0 && id < P.D;
            bx[set] = xn + (long long)(in ? id : 0) * x_plane;
            mx[set] = in ? vx : 0u;
        };
        auto begin_dy = [&](int od) {
            const bool in = od >= 0 && od < P.Do;
            bdy = dyn + (long long)(in ? od : 0) * dy_plane;
            mdy = in ? vdy : 0u;
        };
        auto write_x_piece = [&](int set, int i, char* dst) {
            const bool ok = (mx[set] >> i) & 1;
            uint4 w;
            w.x = ok ? px[set][i].x : 0u; w.y = ok ? px[set][i].y : 0u; w.z = ok ? px[set][i].z : 0u; w.w = ok ? px[set][i].w : 0u;
            if (t + 256 * i < XPIECES) *(uint4*)(dst + lx[i]) = w;
        };
        auto write_dy_piece = [&](int i, char* dst) {
            const bool ok = (mdy >> i) & 1;
            uint4 w;
            w.x = ok ? pdy[i].x : 0u; w.y = ok ? pdy[i].y : 0u; w.z = ok ? pdy[i].z : 0u; w.w = ok ? pdy[i].w : 0u;
            *(uint4*)(dst + ldy[i]) = w;
        };
        // dy planes an x plane needs: tp = id + pD; even tp: od = tp/2 (kd 0) and tp/2 - 1 (kd 2); odd: (tp-1)/2 (kd 1)
        auto floor_half = [](int v) { return (v - (v & 1)) / 2; };  // floor(v / 2) for negative v too

        __syncthreads();
        const int tp0 = id_start + P.pD;
        const bool even0 = (tp0 & 1) == 0;
        {   // first x plane -> LDS (through the set of its parity), second in flight in the other set
            const int m = floor_half(tp0);
            for (int od = m - 1; od <= m; ++od) {
                begin_dy(od);
#pragma unroll
                for (int i = 0; i < NDY; ++i) pdy[i] = *(const uint4*)(bdy + gdy[i]);
#pragma unroll
                for (int i = 0; i < NDY; ++i) write_dy_piece(i, dy_lds + (od & 1) * DY_BYTES);
            }
            begin_dy(m + 1);  // an odd first step writes dy plane m + 1: request it now
#pragma unroll
            for (int i = 0; i < NDY; ++i) pdy[i] = *(const uint4*)(bdy + gdy[i]);
            char* dst = x_lds + (id_start & 1) * X_BYTES;
            if (even0) {
                begin_x(0, id_start);
#pragma unroll
                for (int i = 0; i < NX; ++i) px[0][i] = *(const uint4*)(bx[0] + gx[i]);
#pragma unroll
                for (int i = 0; i < NX; ++i) write_x_piece(0, i, dst);
                begin_x(1, id_start + 1);
#pragma unroll
                for (int i = 0; i < NX; ++i) px[1][i] = *(const uint4*)(bx[1] + gx[i]);
            } else {
                begin_x(1, id_start);
#pragma unroll
                for (int i = 0; i < NX; ++i) px[1][i] = *(const uint4*)(bx[1] + gx[i]);
#pragma unroll
                for (int i = 0; i < NX; ++i) write_x_piece(1, i, dst);
                begin_x(0, id_start + 1);
#pragma unroll
                for (int i = 0; i < NX; ++i) px[0][i] = *(const uint4*)(bx[0] + gx[i]);
            }
        }
        __syncthreads();

        for (int id = id_start; id < id_end; ++id) {
            const int tp = id + P.pD;
            const bool even = (tp & 1) == 0;
            const int m = floor_half(tp);
            const char* x_lane = x_lds + (id & 1) * X_BYTES + x_lane_off;
            char* x_next = x_lds + ((id + 1) & 1) * X_BYTES;
            const char* d0 = dy_lds + (m & 1) * DY_BYTES + coh * DY_SLAB + lane_off;
            const char* d1 = dy_lds + ((m - 1) & 1) * DY_BYTES + coh * DY_SLAB + lane_off;
            const char* const dy_lane[2] = {d0, d1};
            // hook schedule: loads in rows 0..4 (two pieces each), LDS writes in rows 4..8, so that a piece has
            // about a step and a half between its request and its write
            if (even) {
                // set 0 held this plane: refill it with plane id + 2; set 1 (plane id + 1) goes to LDS
                begin_x(0, id + 2);
                begin_dy(m + 1);
                plane_step<true>(acc, x_lane, dy_lane, [&](int r) {
#pragma unroll
                    for (int j = 0; j < 2; ++j) {
                        if (2 * r + j < NX) px[0][2 * r + j] = *(const uint4*)(bx[0] + gx[2 * r + j]);
                        if (r >= 4 && 2 * (r - 4) + j < NX) write_x_piece(1, 2 * (r - 4) + j, x_next);
                    }
                    if (r < NDY) pdy[r] = *(const uint4*)(bdy + gdy[r]);
                });
            } else {
                char* dy_next = dy_lds + ((m + 1) & 1) * DY_BYTES;
                begin_x(1, id + 2);
                plane_step<false>(acc, x_lane, dy_lane, [&](int r) {
#pragma unroll
                    for (int j = 0; j < 2; ++j) {
                        if (2 * r + j < NX) px[1][2 * r + j] = *(const uint4*)(bx[1] + gx[2 * r + j]);
                        if (r >= 4 && 2 * (r - 4) + j < NX) write_x_piece(0, 2 * (r - 4) + j, x_next);
                    }
                    if (r >= XR - NDY) write_dy_piece(r - (XR - NDY), dy_next);  // requested during the previous even step (or before the loop)
                });
            }
            __syncthreads();
        }
    }

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

bool wgrad_s2_supported(const Geom& g) {
    if (g.dtype != MI3D_BF16 || g.kD != 3 || g.kH != 3 || g.kW != 3) return false;
    if (g.sD != 2 || g.sH != 2 || g.sW != 2) return false;
    if (g.pD > 1 || g.pH > 1 || g.pW > 1) return false;
    return g.Cin % 32 == 0 && g.Cout % 32 == 0;
}

static int wgrad_s2_slots(const Geom& g) {
    long long pairs = (long long)(g.Cin / 32) * (g.Cout / 32);
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
    P.CoT = g.Cout / 32;
    P.units = (long long)g.N * P.HT * P.WT * g.D;
    P.slots = wgrad_s2_slots(g);
    const int pairs = P.CiT * P.CoT;
    if (pairs > 65535) return MI3D_ERR_UNSUPPORTED;
    const size_t lds = 2 * X_BYTES + 2 * DY_BYTES;
    static bool attr_set = false;
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute((const void*)wgrad_s2_kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) { note_hip_error(e); return MI3D_ERR_HIP; }
        attr_set = true;
    }
    wgrad_s2_kernel<<<dim3((unsigned)P.slots, (unsigned)pairs), 256, lds, s>>>(P);
    int st = check_launch();
    if (st) return st;
    long long n = g.w_elems();
    return reduce_partials((const float*)ws, dw, n, P.slots, s);
}

}  // namespace mi3d
