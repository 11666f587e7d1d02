// fp32 convolution on the fp32 matrix cores (v_mfma_f32_32x32x2_f32): forward, data gradient and weight gradient of
// the feature-map layers of Section 3.1 for any kernel extent up to 3 and stride up to 2, the precision the paper's
// own runs presumably used (Section 4.1 names none).
//
// Forward pass and data gradient are one kernel, a "gather convolution" over an iteration space j:
//     out[n, os * j + oo, m] = sum over taps t and channels k of  in[n, is * j + delta_t, k] * wt[t][k][m]
// per axis.  The forward pass has is = stride, os = 1, delta_t = t - pad.  The stride-1 data gradient reads dy with
// delta_t = pad - t and the weights with their channel roles swapped.  The stride-2 data gradient is split into the 8
// parity classes of the output position: class pi writes positions 2 j + pi and sees the taps t with pi + pad - t
// even, at delta_t = (pi + pad - t) / 2, so no product with a structural zero is formed.  The 2x2x2 stride-2
// up-sampling layers (run as the data gradient of a 2x2x2 / stride-2 convolution) are the same thing with one tap per
// class.
// MFMA roles: A = weights (M = 32 output channels, K = 2 contracted channels), B = input (N = 32 positions along W),
// so a lane ends with 16 output channels of one position.  A workgroup (4 waves) owns 8 rows x 32 columns of one j
// plane for 32 or 64 output channels and stages, per group of taps that share an input plane and per chunk of the
// contracted channels, the input patch with halo and the group's weights in LDS.  An fp32 MFMA takes 64 cycles and
// needs 8 bytes of operands per lane, so plain 4-byte LDS reads keep it fed.
//
// Weight gradient: contraction over positions, A = dy (M = 32 output channels, K = 2 neighbouring positions along W),
// B = x at the tap's shift (N = 32 input channels); a workgroup owns one 32 x 32 block of (cout, cin) for all taps
// (dealt round-robin to its 8 waves) over a range of position tiles; per-workgroup partial sums are added in index
// order by reduce_partials (bit-reproducible).
#include "mi3d_internal.h"

namespace mi3d {
namespace {

typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;

// j tile of a workgroup: 256 positions, 8 rows x 32 columns or 16 x 16 (whichever covers the plane with fewer positions
// outside it: 48 columns are 3 x 16 but 2 x 32 with a quarter wasted, 12 x 12 fits one 16 x 16 tile).  A wave owns two
// MFMA blocks of 32 positions; position f of the tile is row f / TJW, column f % TJW.
constexpr int MAX_TAPS = 27;
// Waves of a convolution workgroup with 32 / 64 output channels.  With 64 channels eight waves take one block of 32
// positions each (72 registers instead of 107: six or seven waves per SIMD instead of four; strided forward 2.90 ->
// 2.44 ms at 192^3, the stride-1 layers 1 % faster); with 32 channels four waves of two blocks stay (eight: 96 instead
// of 103 TFLOP/s, every weight read then feeds one MFMA instead of two).
constexpr int GC_NW1 = 4, GC_NW2 = 8;
// Budget for the tiles of a stage.  40 KB makes a stage 8 contracted channels deep for the 3x3x3 layers (21 KB with
// 32 output channels per workgroup, 31 KB with 64), so that several workgroups share a CU and one's staging hides behind
// the others' MFMAs: 64->32 at 192^3 93 -> 106 TFLOP/s, 128->64 at 96^3 98 -> 112 (64 KB: 16 channels; 20 KB: 4
// channels, slower again: 92 and 100).
constexpr int LDS_SOFT = 40 * 1024;
constexpr int LDS_SOFT_STRIDED = 64 * 1024;   // forward passes with stride 2

struct GcParams {
    const float* in; const float* in2;     // input (second half of the channels of a virtually concatenated input)
    float* out; float* out2;               // output (second half of the channels of an output written as two tensors)
    const float* wpack;                    // [tap][K][Mpad] weights, M fastest, zero beyond M
    const float* ref; const float* add;    // optional epilogue operands of the output's shape (see GcEpilogue)
    float slope;
    int N, Di, Hi, Wi, K;                  // input extents, contracted channels
    int Do, Ho, Wo, M, Mpad;               // output extents, output channels (padded to 32)
    int in_pitch, in_split;                // channels per voxel of each input tensor; first channel that lives in in2
    int out_pitch, out_split;              // same for the output
    int Jd, Jh, Jw, JHT, JWT, MT;          // iteration space, tiles
    int isd, ish, isw, osd, osh, osw, ood, ooh, oow;
    int ntaps, ngroups;
    int gstart[4];                         // taps of group g: gstart[g] .. gstart[g + 1] - 1 (sorted by plane offset)
    int gd[3];                             // input plane offset of each group
    signed char th[MAX_TAPS], tw[MAX_TAPS];  // row / column offsets of each tap
    signed char tapidx[MAX_TAPS];            // its index in the layer's own tap order (slot in wpack)
    int hmin, wmin, prows, pcols;          // smallest offsets; patch extent in LDS
    int TJH, TJW, LW;                      // tile rows, columns (a power of two, 2^LW)
    int flat;                              // 1: row-major tiles over the whole width (TJW = Jw, JWT = 1, JHT = tiles of 256 positions)
    int CK;                                // contracted channels per stage (even)
};

__device__ __forceinline__ f32x16 mfma2(float a, float b, f32x16 c) { return __builtin_amdgcn_mfma_f32_32x32x2f32(a, b, c, 0, 0, 0); }

// The work of one workgroup: tile (n, jd, jht, jwt) of the iteration space, output channel block mt.
// CB = 32-wide blocks of output channels per workgroup
template <int CB, int NW, int NB>
__device__ __forceinline__ void gconv_tile(const GcParams& P, float* lds_f, int n, int jd, int jht, int jwt, int mt) {
    constexpr int NT = 64 * NW;   // threads; NB = blocks of 32 positions per wave (the tile has NW * NB * 32 positions)
    const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
    const int ln = lane & 31, half = lane >> 5;
    const int xp = P.CK + 1;                                   // channel pitch of a staged voxel (odd: no bank conflicts)
    float* xs = lds_f;                                         // [prows][pcols][CK + 1]
    float* ws = lds_f + ((P.prows * P.pcols * xp + 3) & ~3);   // [taps of the group][CK][32 CB]
    const int m0 = mt * 32 * CB;
    // this lane's position in each of the wave's blocks: row and column inside the tile, inside the plane or not;
    // active: the wave has a position inside the plane (its first one; waves without one issue no MFMA)
    int jh0, jw0, tr0, tc0, tr1, tc1;
    bool ok0, ok1, active;
    {
        const int f0 = (NB * wave) * 32 + ln, f1 = NB == 2 ? f0 + 32 : f0;
        if (P.flat) {
            const int base = jht * 256, total = P.Jh * P.Jw;
            jh0 = base / P.Jw; jw0 = 0;
            const int r0 = (base + f0) / P.Jw, r1 = (base + f1) / P.Jw;
            ok0 = base + f0 < total; ok1 = base + f1 < total;
            tr0 = ok0 ? r0 - jh0 : 0; tc0 = ok0 ? base + f0 - r0 * P.Jw : 0;     // (outside: any staged position)
            tr1 = ok1 ? r1 - jh0 : 0; tc1 = ok1 ? base + f1 - r1 * P.Jw : 0;
            active = base + (NB * wave) * 32 < total;
        } else {
            jh0 = jht * P.TJH; jw0 = jwt * P.TJW;
            tr0 = f0 >> P.LW; tc0 = f0 & (P.TJW - 1); tr1 = f1 >> P.LW; tc1 = f1 & (P.TJW - 1);
            ok0 = jh0 + tr0 < P.Jh && jw0 + tc0 < P.Jw; ok1 = jh0 + tr1 < P.Jh && jw0 + tc1 < P.Jw;
            active = jh0 + (((NB * wave) * 32) >> P.LW) < P.Jh;
        }
    }

    f32x16 acc[NB][CB];
#pragma unroll
    for (int r = 0; r < NB; ++r)
#pragma unroll
        for (int cb = 0; cb < CB; ++cb)
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[r][cb][i] = 0.f;

    const long long in_plane = (long long)P.Hi * P.Wi * P.in_pitch;
    for (int c0 = 0; c0 < P.K; c0 += P.CK) {
        const bool hi_in = c0 >= P.in_split;
        const float* src = (hi_in ? P.in2 : P.in) + (long long)n * P.Di * in_plane + (hi_in ? c0 - P.in_split : c0);
        for (int g = 0; g < P.ngroups; ++g) {
            const int id = P.isd * jd + P.gd[g];
            const int t0 = P.gstart[g], nt = P.gstart[g + 1] - t0;
            __syncthreads();   // the previous stage's readers are done
            // ---- input patch: rows ish * jh0 + hmin .., columns isw * jw0 + wmin .., channels c0 .. c0 + CK - 1
            const bool plane_ok = id >= 0 && id < P.Di;
            const int nvox = P.prows * P.pcols;
            if ((P.CK & 3) == 0 && (P.in_pitch & 3) == 0) {
                const int q4 = P.CK >> 2;
                for (int e = t; e < nvox * q4; e += NT) {
                    const int v = e / q4, q = e - v * q4;
                    const int pr = v / P.pcols, pc = v - pr * P.pcols;
                    const int ih = P.ish * jh0 + P.hmin + pr, iw = P.isw * jw0 + P.wmin + pc;
                    float4 val = make_float4(0.f, 0.f, 0.f, 0.f);
                    if (plane_ok && ih >= 0 && ih < P.Hi && iw >= 0 && iw < P.Wi)
                        val = *(const float4*)(src + (long long)id * in_plane + ((long long)ih * P.Wi + iw) * P.in_pitch + 4 * q);
                    float* d = xs + v * xp + 4 * q;
                    d[0] = val.x; d[1] = val.y; d[2] = val.z; d[3] = val.w;
                }
            } else {   // ragged channel counts: element by element, zero beyond K
                for (int e = t; e < nvox * P.CK; e += NT) {
                    const int v = e / P.CK, q = e - v * P.CK;
                    const int pr = v / P.pcols, pc = v - pr * P.pcols;
                    const int ih = P.ish * jh0 + P.hmin + pr, iw = P.isw * jw0 + P.wmin + pc;
                    float val = 0.f;
                    if (plane_ok && c0 + q < P.K && ih >= 0 && ih < P.Hi && iw >= 0 && iw < P.Wi)
                        val = src[(long long)id * in_plane + ((long long)ih * P.Wi + iw) * P.in_pitch + q];
                    xs[v * xp + q] = val;
                }
            }
            // ---- weights of the group's taps: ws[tap][k][m] for m in this workgroup's blocks
            const int wrow = 32 * CB;
            for (int e = t; e < nt * P.CK * (wrow >> 2); e += NT) {
                const int m4 = e % (wrow >> 2);
                const int k = (e / (wrow >> 2)) % P.CK;
                const int tp = e / ((wrow >> 2) * P.CK);
                float4 val = make_float4(0.f, 0.f, 0.f, 0.f);
                if (c0 + k < P.K && m0 + 4 * m4 < P.Mpad)
                    val = *(const float4*)(P.wpack + ((long long)P.tapidx[t0 + tp] * P.K + c0 + k) * P.Mpad + m0 + 4 * m4);
                *(float4*)(ws + (tp * P.CK + k) * wrow + 4 * m4) = val;
            }
            __syncthreads();
            if (!plane_ok) continue;   // zero padding plane: nothing to add (uniform over the workgroup)
            if (!active) continue;     // no block of this wave has a position inside the plane (uniform over the wave)
            // ---- MFMAs: per tap and pair of contracted channels, 2 rows x CB blocks
            for (int tp = 0; tp < nt; ++tp) {
                const int dh = P.th[t0 + tp] - P.hmin, dw = P.tw[t0 + tp] - P.wmin;
                const float* b0 = xs + ((tr0 * P.ish + dh) * P.pcols + tc0 * P.isw + dw) * xp + half;
                const float* b1 = xs + ((tr1 * P.ish + dh) * P.pcols + tc1 * P.isw + dw) * xp + half;
                const float* a = ws + (tp * P.CK + half) * wrow + ln;
                if constexpr (NB == 2) {
#pragma unroll 4
                    for (int kk = 0; kk < P.CK; kk += 2) {
                        const float x0 = b0[kk], x1 = b1[kk];
#pragma unroll
                        for (int cb = 0; cb < CB; ++cb) {
                            const float wv = a[kk * wrow + 32 * cb];
                            acc[0][cb] = mfma2(wv, x0, acc[0][cb]);
                            acc[1][cb] = mfma2(wv, x1, acc[1][cb]);
                        }
                    }
                } else {
#pragma unroll 4
                    for (int kk = 0; kk < P.CK; kk += 2) {
                        const float x0 = b0[kk];
#pragma unroll
                        for (int cb = 0; cb < CB; ++cb) acc[0][cb] = mfma2(a[kk * wrow + 32 * cb], x0, acc[0][cb]);
                    }
                }
            }
        }
    }
    // ---- epilogue: lane (position ln, half) holds output channels 8 (i / 4) + 4 half + i % 4 of each block.
    // The optional operands (second gradient, reference tensor of the derivative) are read 16 bytes at a time (as single
    // floats the stride-2 data gradient with both took 5.5 ms instead of 3.5 at 192^3); a block's operands are
    // requested right where they are used: requesting a whole row's ahead of time costs 15 to 48 registers and, through
    // the lower occupancy, more than it gains.
    const bool vec = (P.out_pitch & 3) == 0;
#pragma unroll
    for (int r = 0; r < NB; ++r) {
        const int jh = jh0 + (r ? tr1 : tr0), jw = jw0 + (r ? tc1 : tc0);
        if (!(r ? ok1 : ok0)) continue;
        const int od = P.osd * jd + P.ood, oh = P.osh * jh + P.ooh, ow = P.osw * jw + P.oow;
        const long long vox = (((long long)n * P.Do + od) * P.Ho + oh) * P.Wo + ow;
#pragma unroll
        for (int cb = 0; cb < CB; ++cb)
#pragma unroll
            for (int g4 = 0; g4 < 4; ++g4) {
                int c = m0 + 32 * cb + 8 * g4 + 4 * half;
                if (c >= P.M) continue;
                float v[4] = {acc[r][cb][4 * g4], acc[r][cb][4 * g4 + 1], acc[r][cb][4 * g4 + 2], acc[r][cb][4 * g4 + 3]};
                const bool hi_out = c >= P.out_split;
                float* dst = (hi_out ? P.out2 : P.out) + vox * P.out_pitch + (hi_out ? c - P.out_split : c);
                const long long eoff = vox * P.out_pitch + (hi_out ? c - P.out_split : c);   // same offset in ref / add (never split)
                const int nv = P.M - c < 4 ? P.M - c : 4;
                if (vec && nv == 4) {
                    const float4 a4 = P.add ? *(const float4*)(P.add + eoff) : make_float4(0.f, 0.f, 0.f, 0.f);
                    const float4 r4 = P.ref ? *(const float4*)(P.ref + eoff) : make_float4(0.f, 0.f, 0.f, 0.f);
                    const float ad[4] = {a4.x, a4.y, a4.z, a4.w};
                    const float rf[4] = {r4.x, r4.y, r4.z, r4.w};
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        float x = v[i];
                        if (P.add) x += ad[i];
                        if (P.ref) x = rf[i] > 0.f ? x : P.slope * x;
                        else x = x > 0.f ? x : P.slope * x;
                        v[i] = x;
                    }
                    *(float4*)dst = make_float4(v[0], v[1], v[2], v[3]);
                    continue;
                }
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    if (i >= nv) break;
                    float x = v[i];
                    if (P.add) x += P.add[eoff + i];
                    if (P.ref) x = P.ref[eoff + i] > 0.f ? x : P.slope * x;
                    else x = x > 0.f ? x : P.slope * x;
                    v[i] = x;
                }
                for (int i = 0; i < nv; ++i) dst[i] = v[i];
            }
    }
}

template <int CB, int NW, int NB>
__global__ void __launch_bounds__(64 * NW, 2) f32_gconv_kernel(GcParams P) {
    extern __shared__ __attribute__((aligned(16))) float lds_f[];
    long long u = blockIdx.x;
    const int mt = (int)(u % P.MT); u /= P.MT;
    const int jwt = (int)(u % P.JWT); u /= P.JWT;
    const int jht = (int)(u % P.JHT); u /= P.JHT;
    const int jd = (int)(u % P.Jd);
    const int n = (int)(u / P.Jd);
    gconv_tile<CB, NW, NB>(P, lds_f, n, jd, jht, jwt, mt);
}

// The parity classes of a stride-2 data gradient in one launch.  Workgroups are dealt to the 8 XCDs by index modulo
// 8, so tile t goes to XCD t % 8 and its classes follow each other there: b = 8 (ncls (t / 8) + class) + t % 8.  The
// classes of a tile read the same input patch, which then comes from that XCD's L2 for all but the first, and
// every XCD gets every class (class = b % 8 would hand each XCD one class).  Used where the classes have the same
// work each.  The grid spans the largest iteration space of the classes; a workgroup whose tile lies
// outside its class's leaves at once.
struct GcMulti {
    GcParams p[8];
    int ncls, MT, JWT, JHT, Jd;
    long long tiles;      // N * Jd * JHT * JWT * MT of the spanning grid
};
static_assert(sizeof(GcMulti) <= 4096, "kernel arguments");

template <int CB, int NW>
__global__ void __launch_bounds__(64 * NW, 2) f32_gconv_classes_kernel(GcMulti Q) {
    extern __shared__ __attribute__((aligned(16))) float lds_f[];
    const long long r = blockIdx.x >> 3;
    const int cls = (int)(r % Q.ncls);
    long long u = (r / Q.ncls) * 8 + (blockIdx.x & 7);
    if (u >= Q.tiles) return;
    const int mt = (int)(u % Q.MT); u /= Q.MT;
    const int jwt = (int)(u % Q.JWT); u /= Q.JWT;
    const int jht = (int)(u % Q.JHT); u /= Q.JHT;
    const int jd = (int)(u % Q.Jd);
    const int n = (int)(u / Q.Jd);
    const GcParams& P = Q.p[cls];
    if (mt >= P.MT || jwt >= P.JWT || jht >= P.JHT || jd >= P.Jd) return;   // (uniform over the workgroup)
    gconv_tile<CB, NW, 8 / NW>(P, lds_f, n, jd, jht, jwt, mt);
}

// wpack[t][k][m] (m padded to Mpad with zeros) from w[co][t][ci]; swap = 0: (k, m) = (ci, co); swap = 1: (k, m) = (co, ci)
__global__ void __launch_bounds__(256) f32_pack_kernel(const float* __restrict__ w, float* __restrict__ wpack, int Cout, int Cin, int T, int Mpad, int swap) {
    const int K = swap ? Cout : Cin, M = swap ? Cin : Cout;
    const long long total = (long long)T * K * Mpad;
    const long long idx = (long long)blockIdx.x * 256 + threadIdx.x;
    if (idx >= total) return;
    const int m = (int)(idx % Mpad);
    const int k = (int)((idx / Mpad) % K);
    const int t = (int)(idx / ((long long)Mpad * K));
    float v = 0.f;
    if (m < M) {
        const int co = swap ? k : m, ci = swap ? m : k;
        v = w[((long long)co * T + t) * Cin + ci];
    }
    wpack[idx] = v;
}

// ---- weight gradient ------------------------------------------------------------------------------------------------
struct WgParams {
    const float* x; const float* x2;   // input (second half of the channels of a virtually concatenated input)
    const float* dy;
    float* part;                       // [split][Cout][T][Cin]
    int N, D, H, W, Cin, Cout, Do, Ho, Wo;
    int kD, kH, kW, sD, sH, sW, pD, pH, pW, T;
    int x_pitch, x_split;
    int TR, TW;                        // output tile: rows, columns (16 or 32)
    int HT, WT, CIT, COT, S;           // tiles per plane, channel blocks, splits
    long long units;                   // N * HT * WT * Do, Do fastest: a workgroup walks along D
    int prows, pcols;                  // staged x patch per plane
    unsigned pcols_magic;              // q / pcols == (q * pcols_magic) >> 16 for every q < prows * pcols (checked on the host)
};

// Waves, threads of a weight-gradient workgroup.  Eight waves share the staged tiles and take 3 or 4 taps each (64
// accumulator registers instead of 112 with four waves), so two workgroups per CU are four waves per SIMD: 91 -> 100
// TFLOP/s on the 192^3 layers.  Sixteen waves in one workgroup per CU: 88 (no second workgroup to compute while this
// one stages).
constexpr int WG_NW = 8, WG_NT = 64 * WG_NW;

// A workgroup walks a contiguous range of (sample, tile, output plane) units with the output plane running fastest, so
// consecutive units share input planes: the kD planes a unit needs live in a ring of kD LDS slots (plane id in slot
// id mod kD) and only the planes that were not there for the previous unit are fetched.
__global__ void __launch_bounds__(WG_NT, 2) f32_wgrad_kernel(WgParams P) {
    extern __shared__ __attribute__((aligned(16))) float lds_f[];
    const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
    const int ln = lane & 31, half = lane >> 5;
    constexpr int CP = 32;                                     // channels per staged voxel (reads run along the channels)
    float* dys = lds_f;                                        // [TR][TW][32]
    float* xs = lds_f + P.TR * P.TW * CP;                      // [kD ring][prows][pcols][32]
    const int pv = P.prows * P.pcols;
    int b = blockIdx.x;
    const int split = b % P.S; b /= P.S;
    const int cit = b % P.CIT;
    const int cot = b / P.CIT;
    const int ci0 = cit * 32, co0 = cot * 32;
    const bool hi_x = ci0 >= P.x_split;
    const float* xsrc = (hi_x ? P.x2 : P.x) + (hi_x ? ci0 - P.x_split : ci0);
    const bool vec_x = (P.x_pitch & 3) == 0 && (P.Cin & 3) == 0, vec_dy = (P.Cout & 3) == 0;

    constexpr int MAXA = (27 + WG_NW - 1) / WG_NW;   // taps per wave: 27 taps dealt round-robin to the waves
    f32x16 acc[MAXA];
#pragma unroll
    for (int a = 0; a < MAXA; ++a)
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[a][i] = 0.f;

    const long long u0 = P.units * split / P.S, u1 = P.units * (split + 1) / P.S;
    const long long x_plane = (long long)P.H * P.W * P.x_pitch;
    const int c4 = t & 7, vslot = t >> 3;   // staging: 8 threads x 16 bytes per voxel, WG_NT / 8 voxels per pass
    long long cur_col = -1;
    int have_lo = 1, have_hi = 0;           // input planes resident in the ring (none)
    for (long long u = u0; u < u1; ++u) {
        const long long col = u / P.Do;
        const int od = (int)(u - col * P.Do);
        long long r = col;
        const int wt = (int)(r % P.WT); r /= P.WT;
        const int ht = (int)(r % P.HT);
        const int n = (int)(r / P.HT);
        const int oh0 = ht * P.TR, ow0 = wt * P.TW;
        if (col != cur_col) { cur_col = col; have_lo = 1; have_hi = 0; }
        const int need_lo = od * P.sD - P.pD, need_hi = need_lo + P.kD - 1;
        __syncthreads();   // every wave is done with the previous unit's tiles
        // ---- dy tile: TR rows x TW columns x 32 output channels (zero outside the tensor)
        if (vec_dy) {
            for (int v = vslot; v < P.TR * P.TW; v += WG_NT / 8) {
                const int tr = v / P.TW, tc = v - tr * P.TW;
                const int oh = oh0 + tr, ow = ow0 + tc;
                float4 val = make_float4(0.f, 0.f, 0.f, 0.f);
                if (oh < P.Ho && ow < P.Wo && co0 + 4 * c4 < P.Cout)
                    val = *(const float4*)(P.dy + ((((long long)n * P.Do + od) * P.Ho + oh) * P.Wo + ow) * P.Cout + co0 + 4 * c4);
                *(float4*)(dys + v * CP + 4 * c4) = val;
            }
        } else {
            for (int e = t; e < P.TR * P.TW * 32; e += WG_NT) {
                const int c = e & 31, v = e >> 5;
                const int tr = v / P.TW, tc = v - tr * P.TW;
                const int oh = oh0 + tr, ow = ow0 + tc;
                float val = 0.f;
                if (oh < P.Ho && ow < P.Wo && co0 + c < P.Cout)
                    val = P.dy[((((long long)n * P.Do + od) * P.Ho + oh) * P.Wo + ow) * P.Cout + co0 + c];
                dys[v * CP + c] = val;
            }
        }
        // ---- x patches: rows oh0 sH - pH .., columns ow0 sW - pW .., 32 input channels, of the planes not yet in the ring
        for (int id = need_lo; id <= need_hi; ++id) {
            if (id >= have_lo && id <= have_hi) continue;
            float* dst = xs + (((id % P.kD) + P.kD) % P.kD) * pv * CP;
            const bool plane_ok = id >= 0 && id < P.D;
            const float* src = xsrc + ((long long)n * P.D + (plane_ok ? id : 0)) * x_plane;
            if (vec_x) {
                for (int q = vslot; q < pv; q += WG_NT / 8) {
                    const int pr = (int)(((unsigned)q * P.pcols_magic) >> 16), pc = q - pr * P.pcols;
                    const int ih = oh0 * P.sH - P.pH + pr, iw = ow0 * P.sW - P.pW + pc;
                    float4 val = make_float4(0.f, 0.f, 0.f, 0.f);
                    if (plane_ok && ih >= 0 && ih < P.H && iw >= 0 && iw < P.W && ci0 + 4 * c4 < P.Cin)
                        val = *(const float4*)(src + ((long long)ih * P.W + iw) * P.x_pitch + 4 * c4);
                    *(float4*)(dst + q * CP + 4 * c4) = val;
                }
            } else {
                for (int e = t; e < pv * 32; e += WG_NT) {
                    const int c = e & 31, q = e >> 5;
                    const int pr = (int)(((unsigned)q * P.pcols_magic) >> 16), pc = q - pr * P.pcols;
                    const int ih = oh0 * P.sH - P.pH + pr, iw = ow0 * P.sW - P.pW + pc;
                    float val = 0.f;
                    if (plane_ok && ih >= 0 && ih < P.H && iw >= 0 && iw < P.W && ci0 + c < P.Cin)
                        val = src[((long long)ih * P.W + iw) * P.x_pitch + c];
                    dst[q * CP + c] = val;
                }
            }
        }
        have_lo = need_lo; have_hi = need_hi;
        __syncthreads();
        // ---- this wave's taps: K runs over pairs of neighbouring output columns
#pragma unroll
        for (int a = 0; a < MAXA; ++a) {
            const int tap = wave + WG_NW * a;
            if (tap >= P.T) break;
            const int kw = tap % P.kW, kh = (tap / P.kW) % P.kH, kd = tap / (P.kW * P.kH);
            const int id = need_lo + kd;
            const float* plane = xs + (((id % P.kD) + P.kD) % P.kD) * pv * CP;
            for (int tr = 0; tr < P.TR; ++tr) {
                const float* ap = dys + (tr * P.TW + half) * CP + ln;
                const float* bp = plane + ((tr * P.sH + kh) * P.pcols + half * P.sW + kw) * CP + ln;
#pragma unroll 4
                for (int c2 = 0; c2 < P.TW; c2 += 2)
                    acc[a] = mfma2(ap[c2 * CP], bp[c2 * P.sW * CP], acc[a]);
            }
        }
    }
    // ---- partial sums: lane holds input channel ci0 + ln, output channels co0 + 8 (i / 4) + 4 half + i % 4
    float* part = P.part + (long long)split * P.Cout * P.T * P.Cin;
#pragma unroll
    for (int a = 0; a < MAXA; ++a) {
        const int tap = wave + WG_NW * a;
        if (tap >= P.T) break;
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            const int co = co0 + 8 * (i >> 2) + 4 * half + (i & 3), ci = ci0 + ln;
            if (co < P.Cout && ci < P.Cin) part[((long long)co * P.T + tap) * P.Cin + ci] = acc[a][i];
        }
    }
}

// Weight gradient of a 3x3x3 / stride-1 layer with at most 4 input channels (the network's first layer).  The general
// kernel above would give each tap a 32 x 32 block of which 4 columns are in use; here (tap, input channel) pairs are
// the columns: four groups of 8 taps x 4 channels, one group and one block per wave (27 taps: the last group has 3).
// Lane column ln of wave w is tap 8 w + ln / 4, channel ln % 4, so the B operand is a per-lane shifted read of the
// staged x patch ([plane ring][row][column][4 channels]); units, ring and partial sums as in the general kernel.
__global__ void __launch_bounds__(256, 2) f32_wgrad_c4_kernel(WgParams P) {
    extern __shared__ __attribute__((aligned(16))) float lds_f[];
    const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
    const int ln = lane & 31, half = lane >> 5;
    float* dys = lds_f;                                        // [TR][TW][32 output channels]
    float* xs = lds_f + P.TR * P.TW * 32;                      // [3 ring slots][prows][pcols][4]
    const int pv = P.prows * P.pcols;
    const int split = blockIdx.x % P.S, cot = blockIdx.x / P.S;
    const int co0 = cot * 32;
    const int tap = 8 * wave + (ln >> 2), ci = ln & 3;
    const bool col_ok = tap < 27 && ci < P.Cin;
    const int kd = tap / 9, kh = (tap / 3) % 3, kw = tap % 3;   // (tap >= 27: reads inside the staged patch, value unused)
    f32x16 acc[2];
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[a][i] = 0.f;

    const long long u0 = P.units * split / P.S, u1 = P.units * (split + 1) / P.S;
    const long long x_plane = (long long)P.H * P.W * P.Cin;
    const int c4 = t & 7, vslot = t >> 3;   // dy staging: 8 threads x 16 bytes per voxel, 32 voxels per pass
    long long cur_col = -1;
    int have_lo = 1, have_hi = 0;           // input planes resident in the ring (none)
    for (long long u = u0; u < u1; ++u) {
        const long long col = u / P.Do;
        const int od = (int)(u - col * P.Do);
        long long r = col;
        const int wt = (int)(r % P.WT); r /= P.WT;
        const int ht = (int)(r % P.HT);
        const int n = (int)(r / P.HT);
        const int oh0 = ht * P.TR, ow0 = wt * P.TW;
        if (col != cur_col) { cur_col = col; have_lo = 1; have_hi = 0; }
        const int need_lo = od - P.pD, need_hi = need_lo + 2;
        __syncthreads();   // every wave is done with the previous unit's tiles
        for (int v = vslot; v < P.TR * P.TW; v += 32) {
            const int tr = v / P.TW, tc = v - tr * P.TW;
            const int oh = oh0 + tr, ow = ow0 + tc;
            float4 val = make_float4(0.f, 0.f, 0.f, 0.f);
            if (oh < P.Ho && ow < P.Wo && co0 + 4 * c4 < P.Cout)
                val = *(const float4*)(P.dy + ((((long long)n * P.Do + od) * P.Ho + oh) * P.Wo + ow) * P.Cout + co0 + 4 * c4);
            *(float4*)(dys + v * 32 + 4 * c4) = val;
        }
        for (int id = need_lo; id <= need_hi; ++id) {
            if (id >= have_lo && id <= have_hi) continue;
            float* dst = xs + ((id % 3 + 3) % 3) * pv * 4;
            const bool plane_ok = id >= 0 && id < P.D;
            const float* src = P.x + ((long long)n * P.D + (plane_ok ? id : 0)) * x_plane;
            for (int q = t; q < pv; q += 256) {
                const int pr = q / P.pcols, pc = q - pr * P.pcols;
                const int ih = oh0 - P.pH + pr, iw = ow0 - P.pW + pc;
                float4 val = make_float4(0.f, 0.f, 0.f, 0.f);
                if (plane_ok && ih >= 0 && ih < P.H && iw >= 0 && iw < P.W) {
                    const float* px = src + ((long long)ih * P.W + iw) * P.Cin;
                    if (P.Cin == 4) val = *(const float4*)px;
                    else { val.x = px[0]; if (P.Cin > 1) val.y = px[1]; if (P.Cin > 2) val.z = px[2]; }
                }
                *(float4*)(dst + q * 4) = val;
            }
        }
        have_lo = need_lo; have_hi = need_hi;
        __syncthreads();
        const float* plane = xs + (((need_lo + kd) % 3 + 3) % 3) * pv * 4 + ci;
        for (int tr = 0; tr < P.TR; ++tr) {
            const float* ap = dys + (tr * P.TW + half) * 32 + ln;
            const float* bp = plane + ((tr + kh) * P.pcols + half + kw) * 4;
#pragma unroll 4
            for (int c2 = 0; c2 < P.TW; c2 += 4) {   // K = pairs of neighbouring output columns, two chains
                const float b0 = bp[c2 * 4], b1 = bp[(c2 + 2) * 4];
                acc[0] = mfma2(ap[c2 * 32], col_ok ? b0 : 0.f, acc[0]);
                acc[1] = mfma2(ap[(c2 + 2) * 32], col_ok ? b1 : 0.f, acc[1]);
            }
        }
    }
    // partial sums: lane column (tap, ci), rows are the output channels co0 + 8 (i / 4) + 4 half + i % 4
    float* part = P.part + (long long)split * P.Cout * 27 * P.Cin;
#pragma unroll
    for (int i = 0; i < 16; ++i) {
        const int co = co0 + 8 * (i >> 2) + 4 * half + (i & 3);
        if (col_ok && co < P.Cout) part[((long long)co * 27 + tap) * P.Cin + ci] = acc[0][i] + acc[1][i];
    }
}

int cu_count() {
    int dev = 0, cus = 256;
    if (hipGetDevice(&dev) == hipSuccess) (void)hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev);
    return cus;
}

// one axis of the gather convolution: valid taps of a class and their input offsets
struct AxisTaps { int n; int t[3]; int d[3]; };

// forward: every tap, delta = t - p.  data gradient, stride 1: every tap, delta = p - t.  data gradient, stride 2,
// class pi: taps with pi + p - t even, delta = (pi + p - t) / 2 (floor division is exact here, also for negatives)
AxisTaps axis_taps(int k, int s, int p, bool dgrad, int pi) {
    AxisTaps a{0, {0, 0, 0}, {0, 0, 0}};
    for (int t = 0; t < k; ++t) {
        if (!dgrad) { a.t[a.n] = t; a.d[a.n++] = t - p; continue; }
        const int v = pi + p - t;
        if (v % s) continue;
        a.t[a.n] = t; a.d[a.n++] = v / s;
    }
    return a;
}

size_t pack_bytes(const Geom& g, int pass) {
    const int K = pass == MI3D_PASS_DGRAD ? g.Cout : g.Cin, M = pass == MI3D_PASS_DGRAD ? g.Cin : g.Cout;
    const int Mpad = (M + 31) / 32 * 32;
    return ((size_t)g.taps() * K * Mpad * sizeof(float) + 255) & ~(size_t)255;
}

void wgrad_layout(const Geom& g, WgParams* P) {
    P->TR = 2;
    P->TW = (g.sW == 1) ? 32 : 16;
    // (2x2x2 stride 2: one tap per wave and 16 MFMAs per tile and wave leave the kernel waiting for its staging; 32 columns
    // double the work per staged tile, and the x patch of two planes still leaves room for two workgroups per CU)
    if (g.sW == 2 && g.kD <= 2 && g.kH <= 2 && g.kW <= 2 && g.Wo % 32 == 0) P->TW = 32;   // (1.43 -> 1.27 ms at 192^3)
    // Stride 1.  Width: 32 columns, 16 where that leaves fewer positions outside the plane (48 = 3 x 16 columns); planes
    // narrower than 32 take their own (even) width: the contraction runs over pairs of neighbouring columns, so any
    // even width works (24^3 layers 70 -> 88 TFLOP/s).  Rows: as many as make about 96 positions (3 x 32, 6 x 16,
    // 4 x 24) while the dy tile and the ring of x planes leave room for two workgroups per CU (78 KB each), fewer
    // where that divides the height better: more MFMAs per staged tile and fewer halo rows per row (2 x 32 -> 3 x 32:
    // 100 -> 106 TFLOP/s on the 192^3 layers).
    auto padded = [&](int tr, int tw) { return (long long)((g.Ho + tr - 1) / tr * tr) * ((g.Wo + tw - 1) / tw * tw); };
    if (g.sW == 1) {
        if (g.Wo < 32) P->TW = (g.Wo + 1) & ~1;
        else if (padded(2, 16) < padded(2, 32)) P->TW = 16;
        auto lds = [&](int tr) { return ((size_t)tr * P->TW + (size_t)g.kD * ((tr - 1) * g.sH + g.kH) * ((P->TW - 1) * g.sW + g.kW)) * 32 * sizeof(float); };
        int tr = 96 / P->TW;
        tr = tr < 2 ? 2 : (tr > 8 ? 8 : tr);
        while (tr > 2 && (lds(tr) > 78 * 1024 || padded(tr, P->TW) > padded(tr - 1, P->TW))) --tr;
        P->TR = tr;
    }
    P->prows = (P->TR - 1) * g.sH + g.kH;
    P->pcols = (P->TW - 1) * g.sW + g.kW;
    P->pcols_magic = 65536u / (unsigned)P->pcols + 1u;
    P->HT = (g.Ho + P->TR - 1) / P->TR;
    P->WT = (g.Wo + P->TW - 1) / P->TW;
    P->CIT = (g.Cin + 31) / 32;
    P->COT = (g.Cout + 31) / 32;
    P->units = (long long)g.N * g.Do * P->HT * P->WT;
    // about four workgroups per CU in all, each with at least a few units to walk
    long long s = 4ll * cu_count() / ((long long)P->CIT * P->COT);
    if (s > P->units / 4) s = P->units / 4;
    if (s > 1024) s = 1024;
    if (s < 1) s = 1;
    P->S = (int)s;
}

// the folded-tap kernel for at most 4 input channels: 4 x 32 output tiles, two workgroups per CU
bool wgrad_c4_ok(const Geom& g) {
    return g.kD == 3 && g.kH == 3 && g.kW == 3 && g.sD == 1 && g.sH == 1 && g.sW == 1 && g.Cin <= 4 && g.Cout % 4 == 0 && !g.hi;
}
void wgrad_c4_layout(const Geom& g, WgParams* P) {
    P->TR = 4;
    P->TW = 32;
    P->prows = P->TR + 2;
    P->pcols = P->TW + 2;
    P->pcols_magic = 0;
    P->HT = (g.Ho + P->TR - 1) / P->TR;
    P->WT = (g.Wo + P->TW - 1) / P->TW;
    P->CIT = 1;
    P->COT = (g.Cout + 31) / 32;
    P->units = (long long)g.N * g.Do * P->HT * P->WT;
    long long s = 2ll * cu_count() / P->COT;
    if (s > P->units / 4) s = P->units / 4;
    if (s > 1024) s = 1024;
    if (s < 1) s = 1;
    P->S = (int)s;
}

bool wgrad_magic_ok(const WgParams& P) {
    for (unsigned q = 0; q < (unsigned)(P.prows * P.pcols); ++q)
        if (((q * P.pcols_magic) >> 16) != q / (unsigned)P.pcols) return false;
    return true;
}

}  // namespace

bool f32_supported(const Geom& g, int pass) {
    if (g.dtype != MI3D_F32) return false;
    if (g.kD > 3 || g.kH > 3 || g.kW > 3 || g.sD > 2 || g.sH > 2 || g.sW > 2) return false;
    if (g.pD > 2 || g.pH > 2 || g.pW > 2) return false;
    // 32-bit offsets inside one sample's plane and sane grids
    if ((long long)g.H * g.W * g.Cin >= (1ll << 30) || (long long)g.Ho * g.Wo * g.Cout >= (1ll << 30)) return false;
    if (g.w_elems() >= (1ll << 28)) return false;
    if (pass == MI3D_PASS_WGRAD) {
        WgParams P;
        wgrad_layout(g, &P);
        const size_t lds = ((size_t)P.TR * P.TW + (size_t)g.kD * P.prows * P.pcols) * 32 * sizeof(float);
        return lds <= 160 * 1024 && (long long)P.CIT * P.COT * P.S < (1ll << 30) && wgrad_magic_ok(P);
    }
    return true;
}

// 1x1x1 layers with a handful of output channels (the segmentation head) run through plain VALU kernels: with 3 of 32
// MFMA rows in use the matrix cores would do ten times the work (measured at 192^3, N = 2: 0.74 / 1.81 / 3.06 ms for the
// three passes on the matrix cores).  A call with an added gradient or a two-tensor operand keeps the general kernel.
static bool f32_head(const Geom& g) { return pointwise_f32_supported(g) && !g.add && !g.hi; }

size_t f32_workspace_bytes(const Geom& g, int pass) {
    if (!f32_supported(g, pass)) return 0;
    size_t b;
    if (pass == MI3D_PASS_WGRAD) {
        WgParams P;
        wgrad_layout(g, &P);
        b = (size_t)P.S * g.w_elems() * sizeof(float);
        if (wgrad_c4_ok(g)) {
            wgrad_c4_layout(g, &P);
            const size_t c = (size_t)P.S * g.w_elems() * sizeof(float);
            b = b > c ? b : c;
        }
    } else {
        b = pack_bytes(g, pass);
    }
    const size_t h = pointwise_f32_workspace_bytes(g, pass);   // (0 where the head kernels do not apply)
    return b > h ? b : h;
}

bool f32_wgrad_folds_taps(const Geom& g) { return f32_supported(g, MI3D_PASS_WGRAD) && wgrad_c4_ok(g); }

bool f32_takes_halves(const Geom& g, int pass) {   // virtual concatenation: halves of Cin in multiples of 32 channels
    return f32_supported(g, pass) && g.Cin % 64 == 0;
}

// 8 x 32 unless 16 x 16 covers the iteration plane with fewer positions outside it; planes narrower than 32 columns in
// row-major order over their whole width (tile k = positions 256 k .. 256 k + 255 of the plane, whatever rows they fall
// in: a 24 x 24 plane is 18 full blocks of 32 positions instead of 24 blocks three quarters full; TJH = the most rows 256
// consecutive positions can touch)
static void gconv_tile_shape(GcParams* P, bool big_tiles) {
    P->flat = P->Jw < 32 ? 1 : 0;
    if (P->flat) {
        P->TJW = P->Jw;
        P->TJH = 255 / P->Jw + 2;
        if (P->TJH > P->Jh) P->TJH = P->Jh;
        P->LW = 0;
        return;
    }
    auto padded = [&](int th, int tw) { return (long long)((P->Jh + th - 1) / th * th) * ((P->Jw + tw - 1) / tw * tw); };
    const bool square = padded(16, 16) < padded(8, 32);
    P->TJH = square ? 16 : 8;
    P->TJW = square ? 16 : 32;
    P->LW = square ? 4 : 5;
    // Layers with at most 32 output channels (one block per workgroup whatever the grid): 16 x 32 tiles for eight waves
    // where they cover the plane as well; the weights of a stage then serve 512 positions and the halo rows are 2 in
    // 18 instead of 2 in 10 (32->32 at 192^3 +2 %).
    if (!square && big_tiles && P->M <= 32 && padded(16, 32) == padded(8, 32)) P->TJH = 16;
}
static int gconv_row_tiles(const GcParams& P) { return P.flat ? (P.Jh * P.Jw + 255) / 256 : (P.Jh + P.TJH - 1) / P.TJH; }
static int gconv_col_tiles(const GcParams& P) { return P.flat ? 1 : (P.Jw + P.TJW - 1) / P.TJW; }

static int gconv_attributes() {
    static std::atomic<bool> attr_set{false};   // set once per process; a second thread racing here repeats an idempotent call
    if (!attr_set) {
        const void* fns[6] = {(const void*)f32_gconv_kernel<1, GC_NW1, 2>, (const void*)f32_gconv_kernel<2, GC_NW2, 1>, (const void*)f32_gconv_classes_kernel<1, GC_NW1>,
                              (const void*)f32_gconv_classes_kernel<2, GC_NW2>, (const void*)f32_wgrad_kernel, (const void*)f32_gconv_kernel<1, 8, 2>};
        for (const void* f : fns) {
            hipError_t e = hipFuncSetAttribute(f, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
            if (e != hipSuccess) { note_hip_error(e); return MI3D_ERR_HIP; }
        }
        attr_set = true;
    }
    return MI3D_OK;
}

// Output channels per workgroup: 64 where there are that many, unless the grid is so small that its last round
// over the 2 x CUs workgroup slots would be mostly empty and 32-channel workgroups fill the rounds better
// (24^3, N = 2, 256 output channels: 576 workgroups = 2 rounds of 512 at 56 %; 1152 = 3 rounds at 75 %).
// Only where the MFMA work of a workgroup outweighs its staging (taps x contracted channels): a 2x2x2 layer with
// 128 channels got slower with the smaller workgroups (0.40 -> 0.61 ms), which stage the same patch twice.
static int gconv_blocks_of_channels(const GcParams& P, long long tiles, int ntaps) {
    int CB = P.M > 32 ? 2 : 1;
    if (CB == 2 && ntaps * P.K >= 27 * 64) {
        const long long slots = 2ll * cu_count();
        auto fill = [&](int cb) {
            const long long b = tiles * ((P.Mpad + 32 * cb - 1) / (32 * cb));
            return (double)b / (double)(((b + slots - 1) / slots) * slots);
        };
        if (fill(1) > 1.15 * fill(2)) CB = 1;
    }
    return CB;
}

// tiles, channel chunk and LDS bytes of one launch (or one class of a launch) for CB blocks of output channels
static int gconv_prepare(GcParams& P, int CB, size_t* lds) {
    P.JHT = gconv_row_tiles(P);
    P.JWT = gconv_col_tiles(P);
    P.MT = (P.Mpad + 32 * CB - 1) / (32 * CB);
    // contracted channels per stage: the largest even chunk that keeps the tiles of a stage within LDS_SOFT
    int max_group = 1;
    for (int g = 0; g < P.ngroups; ++g) max_group = max_group > P.gstart[g + 1] - P.gstart[g] ? max_group : P.gstart[g + 1] - P.gstart[g];
    auto lds_bytes = [&](int ck) {
        return (size_t)(((P.prows * P.pcols * (ck + 1) + 3) & ~3) + max_group * ck * 32 * CB) * sizeof(float);
    };
    int ck = 32;
    const int kpad = (P.K + 1) & ~1;
    if (ck > kpad) ck = kpad;
    // (strided reads: the patch is four times the tile and the layer is bound by its staging, which deeper stages
    // repeat less often: 32->64 2x2x2 stride 2 at 192^3 1.14 ms with the larger budget, 2.04 with the smaller)
    const size_t soft = (P.isd > 1 || P.ish > 1 || P.isw > 1) ? (size_t)LDS_SOFT_STRIDED : (size_t)LDS_SOFT;
    while (ck > 2 && (lds_bytes(ck) > soft || (kpad % ck && ck > 4))) ck >>= 1;
    if (ck < 2) ck = 2;
    if (lds_bytes(ck) > 160 * 1024) return MI3D_ERR_UNSUPPORTED;
    P.CK = ck;
    *lds = lds_bytes(ck);
    return MI3D_OK;
}

static int launch_gconv(GcParams& P, hipStream_t s) {
    const int CB = gconv_blocks_of_channels(P, (long long)P.N * P.Jd * gconv_row_tiles(P) * gconv_col_tiles(P), P.ntaps);
    size_t lds = 0;
    int st = gconv_prepare(P, CB, &lds);
    if (st) return st;
    const long long blocks = (long long)P.N * P.Jd * P.JHT * P.JWT * P.MT;
    if (blocks <= 0) return MI3D_OK;
    if (blocks > 0x7fffffffll) return MI3D_ERR_UNSUPPORTED;
    if ((st = gconv_attributes())) return st;
    if (CB == 2) f32_gconv_kernel<2, GC_NW2, 1><<<(unsigned)blocks, 64 * GC_NW2, lds, s>>>(P);
    else if (P.TJH == 16 && P.TJW == 32) f32_gconv_kernel<1, 8, 2><<<(unsigned)blocks, 512, lds, s>>>(P);   // 512 positions
    else f32_gconv_kernel<1, GC_NW1, 2><<<(unsigned)blocks, 64 * GC_NW1, lds, s>>>(P);
    return check_launch();
}

// all classes of a stride-2 data gradient in one launch (Q.p[0 .. ncls - 1] filled in but for tiles, CK)
static int launch_gconv_classes(GcMulti& Q, hipStream_t s) {
    if (Q.ncls == 0) return MI3D_OK;
    long long tiles = 0;
    int ntaps = 0;
    for (int c = 0; c < Q.ncls; ++c) {
        const GcParams& P = Q.p[c];
        const long long tc = (long long)P.N * P.Jd * gconv_row_tiles(P) * gconv_col_tiles(P);
        tiles += tc;
        ntaps = ntaps > P.ntaps ? ntaps : P.ntaps;
    }
    const int CB = gconv_blocks_of_channels(Q.p[0], tiles, ntaps);
    size_t lds = 0;
    Q.MT = Q.JWT = Q.JHT = Q.Jd = 0;
    for (int c = 0; c < Q.ncls; ++c) {
        size_t l = 0;
        int st = gconv_prepare(Q.p[c], CB, &l);
        if (st) return st;
        lds = lds > l ? lds : l;
        Q.MT = Q.MT > Q.p[c].MT ? Q.MT : Q.p[c].MT;
        Q.JWT = Q.JWT > Q.p[c].JWT ? Q.JWT : Q.p[c].JWT;
        Q.JHT = Q.JHT > Q.p[c].JHT ? Q.JHT : Q.p[c].JHT;
        Q.Jd = Q.Jd > Q.p[c].Jd ? Q.Jd : Q.p[c].Jd;
    }
    Q.tiles = (long long)Q.p[0].N * Q.Jd * Q.JHT * Q.JWT * Q.MT;
    const long long blocks = (Q.tiles + 7) / 8 * 8 * Q.ncls;
    if (blocks <= 0) return MI3D_OK;
    if (blocks > 0x7fffffffll) return MI3D_ERR_UNSUPPORTED;
    int st = gconv_attributes();
    if (st) return st;
    if (CB == 2) f32_gconv_classes_kernel<2, GC_NW2><<<(unsigned)blocks, 64 * GC_NW2, lds, s>>>(Q);
    else f32_gconv_classes_kernel<1, GC_NW1><<<(unsigned)blocks, 64 * GC_NW1, lds, s>>>(Q);
    return check_launch();
}

// forward (in = x, out = y) and data gradient (in = dy, out = dx)
int f32_conv(const Geom& g, int pass, const void* in, const void* w, void* out, void* ws, size_t ws_bytes, hipStream_t s) {
    if (f32_head(g)) return pointwise_f32_conv(g, pass, in, w, out, ws, ws_bytes, s);
    if (ws_bytes < f32_workspace_bytes(g, pass)) return MI3D_ERR_WORKSPACE;
    const bool dgrad = pass == MI3D_PASS_DGRAD;
    const int T = (int)g.taps();
    const int K = dgrad ? g.Cout : g.Cin, M = dgrad ? g.Cin : g.Cout, Mpad = (M + 31) / 32 * 32;
    const long long total = (long long)T * K * Mpad;
    f32_pack_kernel<<<(unsigned)((total + 255) / 256), 256, 0, s>>>((const float*)w, (float*)ws, g.Cout, g.Cin, T, Mpad, dgrad ? 1 : 0);
    int st = check_launch();
    if (st) return st;
    GcParams B;
    B.in = B.in2 = (const float*)in;
    B.out = B.out2 = (float*)out;
    B.ref = (const float*)g.ref;
    B.add = (const float*)g.add;
    B.slope = g.slope;
    B.N = g.N; B.K = K; B.M = M; B.Mpad = Mpad;
    B.in_pitch = K; B.in_split = 1 << 30; B.out_pitch = M; B.out_split = 1 << 30;
    if (!dgrad) {
        B.Di = g.D; B.Hi = g.H; B.Wi = g.W; B.Do = g.Do; B.Ho = g.Ho; B.Wo = g.Wo;
        if (g.hi) { B.in2 = (const float*)g.hi; B.in_pitch = K / 2; B.in_split = K / 2; }
    } else {
        B.Di = g.Do; B.Hi = g.Ho; B.Wi = g.Wo; B.Do = g.D; B.Ho = g.H; B.Wo = g.W;
        if (g.hi) { B.out2 = (float*)g.hi; B.out_pitch = M / 2; B.out_split = M / 2; }
    }
    const int sD = dgrad ? g.sD : 1, sH = dgrad ? g.sH : 1, sW = dgrad ? g.sW : 1;   // number of classes per axis
    // Classes with the same work each (2x2x2: one tap per class) go into one launch, where they share their input
    // patch through the L2 (192^3, N = 2: 1.74 -> 1.58 ms; 48^3: 0.63 -> 0.30).  Classes of 1 to 8 taps (3x3x3) keep a
    // launch each: merged, their mix left CUs with the eight-tap workgroups behind (6.0 against 5.4 ms).
    const bool classes = sD * sH * sW > 1 && g.kD <= g.sD && g.kH <= g.sH && g.kW <= g.sW;
    GcMulti Q;
    Q.ncls = 0;
    for (int pd = 0; pd < sD; ++pd)
        for (int ph = 0; ph < sH; ++ph)
            for (int pw = 0; pw < sW; ++pw) {
                GcParams P = B;
                const AxisTaps ad = axis_taps(g.kD, g.sD, g.pD, dgrad, pd), ah = axis_taps(g.kH, g.sH, g.pH, dgrad, ph),
                               aw = axis_taps(g.kW, g.sW, g.pW, dgrad, pw);
                if (!dgrad) {
                    P.Jd = g.Do; P.Jh = g.Ho; P.Jw = g.Wo;
                    P.isd = g.sD; P.ish = g.sH; P.isw = g.sW;
                    P.osd = P.osh = P.osw = 1; P.ood = P.ooh = P.oow = 0;
                } else {
                    P.Jd = (g.D - pd + g.sD - 1) / g.sD; P.Jh = (g.H - ph + g.sH - 1) / g.sH; P.Jw = (g.W - pw + g.sW - 1) / g.sW;
                    P.isd = P.ish = P.isw = 1;
                    P.osd = g.sD; P.osh = g.sH; P.osw = g.sW; P.ood = pd; P.ooh = ph; P.oow = pw;
                }
                if (P.Jd <= 0 || P.Jh <= 0 || P.Jw <= 0) continue;
                // taps grouped by input plane offset (the kd axis is the outer one)
                P.ntaps = 0; P.ngroups = 0;
                int hmin = 1 << 20, hmax = -(1 << 20), wmin = 1 << 20, wmax = -(1 << 20);
                for (int a = 0; a < ad.n; ++a) {
                    P.gstart[P.ngroups] = P.ntaps;
                    P.gd[P.ngroups] = ad.d[a];
                    for (int bq = 0; bq < ah.n; ++bq)
                        for (int c = 0; c < aw.n; ++c) {
                            P.th[P.ntaps] = (signed char)ah.d[bq];
                            P.tw[P.ntaps] = (signed char)aw.d[c];
                            P.tapidx[P.ntaps] = (signed char)((ad.t[a] * g.kH + ah.t[bq]) * g.kW + aw.t[c]);
                            hmin = hmin < ah.d[bq] ? hmin : ah.d[bq]; hmax = hmax > ah.d[bq] ? hmax : ah.d[bq];
                            wmin = wmin < aw.d[c] ? wmin : aw.d[c]; wmax = wmax > aw.d[c] ? wmax : aw.d[c];
                            ++P.ntaps;
                        }
                    if (P.ntaps > P.gstart[P.ngroups]) ++P.ngroups;
                }
                P.gstart[P.ngroups] = P.ntaps;
                if (P.ntaps == 0) { hmin = hmax = wmin = wmax = 0; }   // a class no tap reaches: zeros (plus the epilogue)
                P.hmin = hmin; P.wmin = wmin;
                gconv_tile_shape(&P, !classes && sD * sH * sW == 1);
                P.prows = (P.TJH - 1) * P.ish + (hmax - hmin) + 1;
                P.pcols = (P.TJW - 1) * P.isw + (wmax - wmin) + 1;
                P.wpack = (const float*)ws;
                if (classes) { Q.p[Q.ncls++] = P; continue; }
                st = launch_gconv(P, s);
                if (st) return st;
            }
    return classes ? launch_gconv_classes(Q, s) : MI3D_OK;
}

int f32_wgrad(const Geom& g, const void* x, const void* dy, float* dw, void* ws, size_t ws_bytes, hipStream_t s) {
    if (f32_head(g)) return pointwise_f32_conv(g, MI3D_PASS_WGRAD, x, dy, dw, ws, ws_bytes, s);
    if (ws_bytes < f32_workspace_bytes(g, MI3D_PASS_WGRAD)) return MI3D_ERR_WORKSPACE;
    WgParams P;
    wgrad_layout(g, &P);
    P.x = P.x2 = (const float*)x;
    P.dy = (const float*)dy;
    P.part = (float*)ws;
    P.N = g.N; P.D = g.D; P.H = g.H; P.W = g.W; P.Cin = g.Cin; P.Cout = g.Cout; P.Do = g.Do; P.Ho = g.Ho; P.Wo = g.Wo;
    P.kD = g.kD; P.kH = g.kH; P.kW = g.kW; P.sD = g.sD; P.sH = g.sH; P.sW = g.sW; P.pD = g.pD; P.pH = g.pH; P.pW = g.pW;
    P.T = (int)g.taps();
    P.x_pitch = g.Cin; P.x_split = 1 << 30;
    if (g.hi) { P.x2 = (const float*)g.hi; P.x_pitch = g.Cin / 2; P.x_split = g.Cin / 2; }
    if (wgrad_c4_ok(g)) {
        wgrad_c4_layout(g, &P);
        const size_t lds4 = ((size_t)P.TR * P.TW * 32 + (size_t)3 * P.prows * P.pcols * 4) * sizeof(float);   // 26 KB
        f32_wgrad_c4_kernel<<<(unsigned)(P.COT * P.S), 256, lds4, s>>>(P);
        int st4 = check_launch();
        if (st4) return st4;
        return reduce_partials((const float*)ws, dw, g.w_elems(), P.S, s);
    }
    const size_t lds = ((size_t)P.TR * P.TW + (size_t)g.kD * P.prows * P.pcols) * 32 * sizeof(float);
    static std::atomic<bool> attr_set{false};   // set once per process; a second thread racing here repeats an idempotent call
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute((const void*)f32_wgrad_kernel, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
        if (e != hipSuccess) { note_hip_error(e); return MI3D_ERR_HIP; }
        attr_set = true;
    }
    f32_wgrad_kernel<<<(unsigned)(P.CIT * P.COT * P.S), WG_NT, lds, s>>>(P);
    int st = check_launch();
    if (st) return st;
    return reduce_partials((const float*)ws, dw, g.w_elems(), P.S, s);
}

}  // namespace mi3d
