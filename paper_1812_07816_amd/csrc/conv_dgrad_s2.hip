// Data gradient of the 3x3x3 / stride 2 convolution (pad 0 or 1 on every
// axis, Cout <= 64) on bf16 MFMA (v_mfma_f32_32x32x16_bf16), fp32 accumulation:
//   dx[i,ci] = sum over (o,t) with 2 o - p + t == i of sum_co dy[o,co] * w[co,t,ci]
//
// Per axis, input position i = 2 c + e (pair index c, e in {0,1}) receives
//   tap 0 from dy position c + p      and tap 2 from c + p - 1   if i + p is even  ("E")
//   tap 1 from dy position c + p - [p == 1]                      if i + p is odd   ("O")
// so a pair of dx planes / rows / columns needs the two dy positions
// A = c + p - 1 and B = c + p and nothing else: no accumulator is carried from
// one plane pair to the next.  A workgroup owns 4 row pairs (one per wave) x 32
// column pairs and walks along D over plane pairs with a ring of two staged dy
// plane patches (5 x 33 voxels x Cout); all 27 x Cout x 32 weights of its cin
// tile stay in LDS.  Each wave holds the 8 accumulator blocks (plane E/O x row
// E/O x column E/O, 32 cin x 32 column pairs each); the 27 taps are spread over
// them as 8 + 4 + 4 + 4 + 2 + 2 + 2 + 1.  The layer writes 4x the bytes it
// reads, so it is bound by its stores.
#include "mi3d_internal.h"

namespace mi3d {
namespace {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;
typedef __attribute__((__vector_size__(2 * sizeof(float)))) float f32x2;
typedef __attribute__((__vector_size__(2 * sizeof(__bf16)))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(2))) unsigned u32x2;

constexpr int RP = 4, CP = 32;             // row pairs, column pairs per workgroup
constexpr int PR = RP + 1, PC = CP + 1;    // staged dy rows, columns
constexpr int PITCH = 34;                  // row pitch (voxels)
constexpr int SLABV = PR * PITCH;          // voxels per 8-channel slab

struct Dg2Params {
    const uint16_t* dy;
    const uint16_t* wpack;  // [cin tile][kd][kh][kw][k16][lane][8]
    uint16_t* dx;
    uint16_t* dump;         // 8 KB that masked store lanes write to instead of dx
    float* part;            // [cout chunk][voxel][Cin] fp32 partial gradients (Cout > 64)
    const uint16_t* add;    // FUSE: second gradient of dx's shape, added to the rounded result
    const uint16_t* ref;    // FUSE: tensor of dx's shape whose sign selects the factor 1 or slope
    float slope;
    int N, D, H, W, Cin, Cout, Do, Ho, Wo, p;
    int QD, HT, WT, CiT, NCO;   // ..., cin tiles, cout chunks (of 64 when Cout > 64)
    long long units;
    int nwg;
    // FUSE == 2: per-(workgroup, segment, wave) sums of g and g * xhat, 32 cins each, in the layout of the
    // plane-streaming kernel's statistics; key = sample * CiT + cin tile, -1 = unused
    float stat_slope;
    float* stat_part;
    int* stat_key;
    int max_seg;
};

// adds g = v * lrelu'(a) and g * xhat, xhat = lrelu^-1(a), of the 8 packed bf16 values of v (stored gradient) and a
// (activated output of the normalised layer below) to s1[0..7], s2[0..7]; nothing where the lane stores nothing
__device__ __forceinline__ void add_sums8(const uint4& v, const uint4& a, bool ok, float slope, float inv, float* s1, float* s2) {
    const uint32_t vw[4] = {v.x, v.y, v.z, v.w}, aw[4] = {a.x, a.y, a.z, a.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const uint32_t q = ok ? vw[i] : 0u, r = ok ? aw[i] : 0u;
        const float vlo = __builtin_bit_cast(float, q << 16), vhi = __builtin_bit_cast(float, q & 0xffff0000u);
        const float alo = __builtin_bit_cast(float, r << 16), ahi = __builtin_bit_cast(float, r & 0xffff0000u);
        const float glo = alo > 0.f ? vlo : slope * vlo, ghi = ahi > 0.f ? vhi : slope * vhi;
        s1[2 * i] += glo; s2[2 * i] = fmaf(glo, alo > 0.f ? alo : alo * inv, s2[2 * i]);
        s1[2 * i + 1] += ghi; s2[2 * i + 1] = fmaf(ghi, ahi > 0.f ? ahi : ahi * inv, s2[2 * i + 1]);
    }
}

__device__ __forceinline__ f32x16 mfma(bf16x8 a, bf16x8 b, f32x16 c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}

// per-axis tap table for class e (0 = E, 1 = O): number of taps, tap index, source side (0 = A, 1 = B)
template <int P> struct Taps {
    static constexpr int n(int cls) { return cls == 0 ? 2 : 1; }
    static constexpr int tap(int cls, int k) { return cls == 0 ? (k == 0 ? 0 : 2) : 1; }
    static constexpr int side(int cls, int k) { return cls == 0 ? (k == 0 ? 1 : 0) : (P == 1 ? 0 : 1); }
};

// The 27 taps in issue order: accumulator block (cd, ch, cw), weight tap, source fragment (plane, row,
// column side).  Blocks have 8, 4, 4, 4, 2, 2, 2, 1 taps; the order interleaves them (most remaining
// first, never the block just used) so that consecutive MFMAs do not depend on each other.
template <int P> struct TapList {
    int blk[27], tap[27], src[27];
    constexpr TapList() : blk(), tap(), src() {
        int cnt[8] = {}, tp[8][8] = {}, sr[8][8] = {};
        for (int cd = 0; cd < 2; ++cd)
            for (int id = 0; id < Taps<P>::n(cd); ++id)
                for (int ch = 0; ch < 2; ++ch)
                    for (int ih = 0; ih < Taps<P>::n(ch); ++ih)
                        for (int cw = 0; cw < 2; ++cw)
                            for (int iw = 0; iw < Taps<P>::n(cw); ++iw) {
                                const int b = cd * 4 + ch * 2 + cw;
                                tp[b][cnt[b]] = (Taps<P>::tap(cd, id) * 3 + Taps<P>::tap(ch, ih)) * 3 + Taps<P>::tap(cw, iw);
                                sr[b][cnt[b]] = Taps<P>::side(cd, id) * 4 + Taps<P>::side(ch, ih) * 2 + Taps<P>::side(cw, iw);
                                ++cnt[b];
                            }
        int used[8] = {}, prev = -1;
        for (int i = 0; i < 27; ++i) {
            int best = -1;
            for (int b = 0; b < 8; ++b) {
                const int rem = cnt[b] - used[b];
                if (rem > 0 && b != prev && (best < 0 || rem > cnt[best] - used[best])) best = b;
            }
            if (best < 0) best = prev;
            blk[i] = best; tap[i] = tp[best][used[best]]; src[i] = sr[best][used[best]];
            ++used[best]; prev = best;
        }
    }
};

// fp32 block -> packed bf16; lane (n, h) ends with cins 16h .. 16h + 15 of its voxel in two uint4
__device__ __forceinline__ void pack_block(const f32x16& a, uint4 (&c)[2]) {
    uint32_t o[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        f32x2 v = {a[2 * i], a[2 * i + 1]};
        bf16x2 b = __builtin_convertvector(v, bf16x2);
        o[i] = __builtin_bit_cast(uint32_t, b);
    }
#pragma unroll
    for (int k = 0; k < 2; ++k) {
        u32x2 s0 = __builtin_amdgcn_permlane32_swap(o[2 * k], o[2 * k + 4], false, false);
        u32x2 s1 = __builtin_amdgcn_permlane32_swap(o[2 * k + 1], o[2 * k + 5], false, false);
        c[k].x = s0[0]; c[k].y = s1[0]; c[k].z = s0[1]; c[k].w = s1[1];
    }
}

// (v + a) * (m > 0 ? 1 : slope) on packed bf16 pairs: fp32 sum and product, one rounding to nearest even
__device__ __forceinline__ uint32_t fuse_pair(uint32_t v, uint32_t a, uint32_t m, float slope) {
    float lo = __builtin_bit_cast(float, v << 16) + __builtin_bit_cast(float, a << 16);
    float hi = __builtin_bit_cast(float, v & 0xffff0000u) + __builtin_bit_cast(float, a & 0xffff0000u);
    lo = (int)(m << 16) > 0 ? lo : slope * lo;
    hi = (int)(m & 0xffff0000u) > 0 ? hi : slope * hi;
    f32x2 f = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(f, bf16x2));
}
__device__ __forceinline__ uint4 fuse4(uint4 v, uint4 a, uint4 m, float slope) {
    return uint4{fuse_pair(v.x, a.x, m.x, slope), fuse_pair(v.y, a.y, m.y, slope), fuse_pair(v.z, a.z, m.z, slope), fuse_pair(v.w, a.w, m.w, slope)};
}

// KK = Cout / 16 k16 steps.  Every MFMA needs its own 1 KB weight fragment from LDS (a tap is used once
// per wave and step), so the kernel runs at the LDS rate: the fragment reads are issued two groups of
// three MFMAs ahead of their use from a ring of three register groups.
// PART: Cout > 64 is contracted in chunks of 64 that are separate work units writing fp32 partial gradients; a second
// kernel adds the chunks in index order and rounds to bf16.
// FUSE (not with PART): the gradient of a skip connection.  The pieces of G.add and G.ref at the addresses of the
// plane pair's 16 stores are requested before its MFMA work and applied to the rounded result in the store path.
// FUSE == 2: the skip tensor's producer is a normalised layer (Section 4.1), so no factor is applied (G.slope = 1), and
// the kernel adds up the two sums that layer's normalisation needs for its backward pass, from the stored gradient
// and G.ref: every lane keeps the sums of its 16 cins over a segment, a fixed butterfly adds the 32 voxel lanes.
template <int P, int KK, bool PART, int FUSE = 0>
__global__ void __launch_bounds__(256, 1) dgrad_s2_kernel(Dg2Params G) {
    extern __shared__ __attribute__((aligned(16))) char lds[];
    constexpr int SLABS = 2 * KK;
    constexpr int W_BYTES = 27 * KK * 1024;
    constexpr int STAGE = SLABS * SLABV * 16;
    constexpr TapList<P> TL{};
    char* w_lds = lds;
    char* in_lds = lds + W_BYTES;               // two stages, slot = dy plane & 1

    const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
    int g = blockIdx.x;
    if ((G.nwg & 7) == 0) g = (g & 7) * (G.nwg >> 3) + (g >> 3);
    long long u0 = G.units * g / G.nwg, u1 = G.units * (g + 1) / G.nwg;

    const int NPIECE = PR * PC * SLABS;         // 16-byte pieces of a staged plane (<= 1320)
    constexpr int NL = 6;
    int cur_cit = -1;
    int seg_i = 0;   // FUSE == 2: index of the segment within this workgroup's unit range

    while (u0 < u1) {
        long long column = u0 / G.QD;
        const int q_start = (int)(u0 - column * G.QD);
        const long long left = u1 - u0;
        const int q_end = q_start + (int)(left < (long long)(G.QD - q_start) ? left : (long long)(G.QD - q_start));
        u0 += q_end - q_start;
        const int wt = (int)(column % G.WT); column /= G.WT;
        const int ht = (int)(column % G.HT); column /= G.HT;
        const int chunk = PART ? (int)(column % G.NCO) : 0;
        if (PART) column /= G.NCO;
        const int cit = (int)(column % G.CiT);
        const int n = (int)(column / G.CiT);
        const int rq0 = ht * RP, cq0 = wt * CP;   // first row pair / column pair

        __syncthreads();  // previous segment's readers are done
        if (cit * G.NCO + chunk != cur_cit) {
            const uint4* src = (const uint4*)(G.wpack + ((long long)cit * G.NCO + chunk) * (W_BYTES / 2));
            for (int i = t; i < W_BYTES / 16; i += 256) ((uint4*)w_lds)[i] = src[i];
            cur_cit = cit * G.NCO + chunk;
        }
        // load plan: piece q = (voxel v = q / SLABS, slab c = q % SLABS), voxel row-major over 5 x 33
        int goff[NL], loff[NL];
        unsigned valid = 0;
#pragma unroll
        for (int i = 0; i < NL; ++i) {
            const int q = t + 256 * i;
            const int v = q / SLABS, c = q - v * SLABS;
            const int row = v / PC, col = v - row * PC;
            const int gh = rq0 + G.p - 1 + row, gw = cq0 + G.p - 1 + col;
            const bool ok = q < NPIECE && gh >= 0 && gh < G.Ho && gw >= 0 && gw < G.Wo;
            goff[i] = ok ? (gh * G.Wo + gw) * G.Cout + chunk * (16 * KK) + c * 8 : 0;
            loff[i] = (c * SLABV + row * PITCH + col) * 16;
            valid |= (ok ? 1u : 0u) << i;
        }
        const long long dy_plane = (long long)G.Ho * G.Wo * G.Cout;
        const uint16_t* dyn = G.dy + (long long)n * G.Do * dy_plane;
        uint16_t* dxn = G.dx + (long long)n * G.D * G.H * G.W * G.Cin;
        float st1[FUSE == 2 ? 16 : 1], st2[FUSE == 2 ? 16 : 1];
        if constexpr (FUSE == 2) {
#pragma unroll
            for (int i = 0; i < 16; ++i) st1[i] = st2[i] = 0.f;
        }
        const float inv_stat_slope = FUSE == 2 ? 1.f / G.stat_slope : 1.f;
        float* pn = PART ? G.part + ((long long)chunk * G.N + n) * G.D * G.H * G.W * G.Cin : nullptr;

        uint4 pre[NL];
        unsigned pre_mask = 0;
        auto load_plane = [&](int m) {
            const bool in = m >= 0 && m < G.Do;
            const uint16_t* base = dyn + (long long)(in ? m : 0) * dy_plane;
            pre_mask = in ? valid : 0u;
#pragma unroll
            for (int i = 0; i < NL; ++i) pre[i] = *(const uint4*)(base + goff[i]);
        };
        auto write_plane = [&](int slot) {
            char* dst = in_lds + slot * STAGE;
#pragma unroll
            for (int i = 0; i < NL; ++i) {
                const bool ok = (pre_mask >> i) & 1;
                uint4 v;
                v.x = ok ? pre[i].x : 0u; v.y = ok ? pre[i].y : 0u; v.z = ok ? pre[i].z : 0u; v.w = ok ? pre[i].w : 0u;
                if (t + 256 * i < NPIECE) *(uint4*)(dst + loff[i]) = v;
            }
        };

        // planes A = q + p - 1 and B = q + p of the first pair
        load_plane(q_start + G.p - 1);
        write_plane((q_start + G.p - 1) & 1);
        load_plane(q_start + G.p);
        write_plane((q_start + G.p) & 1);
        __syncthreads();

        // per-lane fragment addresses: lane (n = column pair, half h) reads slab 2 kk + h, row wave + side, column n + side
        const int lane_in = ((lane >> 5) * SLABV + wave * PITCH + (lane & 31)) * 16;
        const char* w_lane = w_lds + lane * 16;

        for (int q = q_start; q < q_end; ++q) {
            const int mA = q + G.p - 1, mB = q + G.p;
            load_plane(mB + 1);  // unconditional (after the last pair: a plane nobody reads), so that its wait sits at the LDS write
            const char* plane_base[2] = {in_lds + (mA & 1) * STAGE + lane_in, in_lds + (mB & 1) * STAGE + lane_in};

            // element offsets of this lane's even and odd voxel for block row (cd, ch), -1 outside the tensor
            auto store_offsets = [&](int cd, int ch, long long& oe, long long& oo) {
                const int id_ = 2 * q + (cd == 0 ? G.p : 1 - G.p);
                const int ih_ = 2 * (rq0 + wave) + (ch == 0 ? G.p : 1 - G.p);
                const int iw_ = 2 * (cq0 + (lane & 31));
                const bool row_ok = id_ < G.D && ih_ < G.H;
                const long long o = (((long long)id_ * G.H + ih_) * G.W + iw_) * G.Cin + cit * 32 + 16 * (lane >> 5);
                oe = (row_ok && iw_ < G.W) ? o : -1;
                oo = (row_ok && iw_ + 1 < G.W) ? o + G.Cin : -1;
            };
            uint4 fa[FUSE != 0 ? 4 : 1][4], fm[FUSE != 0 ? 4 : 1][4];   // [cd * 2 + ch][even 0, even 1, odd 0, odd 1]
            if constexpr (FUSE != 0) {
                const long long nbase = (long long)n * G.D * G.H * G.W * G.Cin;
#pragma unroll
                for (int b = 0; b < 4; ++b) {
                    long long oe, oo;
                    store_offsets(b >> 1, b & 1, oe, oo);
                    // unconditional loads: masked lanes read the dump area
                    const uint16_t* ae = oe >= 0 ? G.add + nbase + oe : G.dump + lane * 16;
                    const uint16_t* ao = oo >= 0 ? G.add + nbase + oo : G.dump + lane * 16;
                    const uint16_t* me = oe >= 0 ? G.ref + nbase + oe : G.dump + lane * 16;
                    const uint16_t* mo = oo >= 0 ? G.ref + nbase + oo : G.dump + lane * 16;
                    fa[b][0] = *(const uint4*)ae; fa[b][1] = *(const uint4*)(ae + 8);
                    fa[b][2] = *(const uint4*)ao; fa[b][3] = *(const uint4*)(ao + 8);
                    fm[b][0] = *(const uint4*)me; fm[b][1] = *(const uint4*)(me + 8);
                    fm[b][2] = *(const uint4*)mo; fm[b][3] = *(const uint4*)(mo + 8);
                }
            }

            f32x16 acc[2][2][2];
#pragma unroll
            for (int a = 0; a < 2; ++a)
#pragma unroll
                for (int b = 0; b < 2; ++b)
#pragma unroll
                    for (int c = 0; c < 2; ++c)
#pragma unroll
                        for (int i = 0; i < 16; ++i) acc[a][b][c][i] = 0.f;

            // fragment reads: x of k16 step kk (8 fragments: plane side, row side, column side), weights of MFMA m
            bf16x8 xb[2][8], wq[3][3];
            auto load_x = [&](int kk, int f) {
                xb[kk & 1][f] = *(const bf16x8*)(plane_base[f >> 2] + (2 * kk * SLABV + ((f >> 1) & 1) * PITCH + (f & 1)) * 16);
            };
            auto load_wgroup = [&](int gi) {  // group gi = 3 MFMAs: k16 step gi / 9, list positions 3 (gi % 9) ..
#pragma unroll
                for (int j = 0; j < 3; ++j)
                    wq[gi % 3][j] = *(const bf16x8*)(w_lane + (TL.tap[3 * (gi % 9) + j] * KK + gi / 9) * 1024);
            };
#pragma unroll
            for (int f = 0; f < 8; ++f) load_x(0, f);
            load_wgroup(0);
            load_wgroup(1);
#pragma unroll
            for (int gi = 0; gi < 9 * KK; ++gi) {
                const int kk = gi / 9, grp = gi % 9;
                if (gi + 2 < 9 * KK) load_wgroup(gi + 2);
                if (kk + 1 < KK && grp < 8) load_x(kk + 1, grp);
#pragma unroll
                for (int j = 0; j < 3; ++j) {
                    const int i = 3 * grp + j;
                    f32x16& a = acc[TL.blk[i] >> 2][(TL.blk[i] >> 1) & 1][TL.blk[i] & 1];
                    a = mfma(wq[gi % 3][j], xb[kk & 1][TL.src[i]], a);
                }
                __builtin_amdgcn_sched_barrier(0);
            }

            // stores: dx position of class e on an axis is 2 c + (e == 0 ? p : 1 - p)
            const int cq = cq0 + (lane & 31);
            const int rq = rq0 + wave;
#pragma unroll
            for (int cd = 0; cd < 2; ++cd) {
                const int id_ = 2 * q + (cd == 0 ? G.p : 1 - G.p);
#pragma unroll
                for (int ch = 0; ch < 2; ++ch) {
                    const int ih_ = 2 * rq + (ch == 0 ? G.p : 1 - G.p);
                    if (PART) {
                        // fp32 partials: register i of lane (n, h) is cin 8 (i / 4) + 4 h + i % 4; class cw sits in column
                        // 2 cq + (cw == 0 ? p : 1 - p)
#pragma unroll
                        for (int cw = 0; cw < 2; ++cw) {
                            const int iw_ = 2 * cq + (cw == 0 ? P : 1 - P);
                            float* ptr = pn + (((long long)id_ * G.H + ih_) * G.W + iw_) * G.Cin + cit * 32 + 4 * (lane >> 5);
                            float* qf = (id_ < G.D && ih_ < G.H && iw_ < G.W) ? ptr : (float*)G.dump + lane * 32;
                            const f32x16& a = acc[cd][ch][cw];
#pragma unroll
                            for (int g4 = 0; g4 < 4; ++g4) *(float4*)(qf + 8 * g4) = float4{a[4 * g4], a[4 * g4 + 1], a[4 * g4 + 2], a[4 * g4 + 3]};
                        }
                        continue;
                    }
                    uint4 be[2], bo[2];
                    pack_block(acc[cd][ch][0], be);   // class E columns: 2 cq + p
                    pack_block(acc[cd][ch][1], bo);   // class O columns: 2 cq + 1 - p
                    // even column = E if p == 0 else O
                    uint4 (&ev)[2] = (P == 0) ? be : bo;
                    uint4 (&od)[2] = (P == 0) ? bo : be;
                    // lane (n, h) writes cins 16 h .. 16 h + 15 of the even and of the odd voxel of its column
                    // pair: per store instruction the two lane halves fill 32 of a voxel's 64 bytes (measured:
                    // 5.9 TB/s; giving each lane a whole 64-byte voxel in four 16-byte stores reaches 3.6 TB/s)
                    // Stores are unconditional (masked lanes write to the dump area): behind a branch the compiler
                    // cannot count them and makes the LDS write that follows wait for the stores to complete.
                    const int iw_ = 2 * cq;
                    const bool row_ok = id_ < G.D && ih_ < G.H;
                    uint16_t* ptr = dxn + (((long long)id_ * G.H + ih_) * G.W + iw_) * G.Cin + cit * 32 + 16 * (lane >> 5);
                    uint16_t* pe = (row_ok && iw_ < G.W) ? ptr : G.dump + lane * 16;
                    uint16_t* po = (row_ok && iw_ + 1 < G.W) ? ptr + G.Cin : G.dump + lane * 16;
                    if constexpr (FUSE != 0) {
                        const int b = cd * 2 + ch;
                        ev[0] = fuse4(ev[0], fa[b][0], fm[b][0], G.slope); ev[1] = fuse4(ev[1], fa[b][1], fm[b][1], G.slope);
                        od[0] = fuse4(od[0], fa[b][2], fm[b][2], G.slope); od[1] = fuse4(od[1], fa[b][3], fm[b][3], G.slope);
                        if constexpr (FUSE == 2) {
                            const bool oke = row_ok && iw_ < G.W, oko = row_ok && iw_ + 1 < G.W;
                            add_sums8(ev[0], fm[b][0], oke, G.stat_slope, inv_stat_slope, st1, st2);
                            add_sums8(ev[1], fm[b][1], oke, G.stat_slope, inv_stat_slope, st1 + 8, st2 + 8);
                            add_sums8(od[0], fm[b][2], oko, G.stat_slope, inv_stat_slope, st1, st2);
                            add_sums8(od[1], fm[b][3], oko, G.stat_slope, inv_stat_slope, st1 + 8, st2 + 8);
                        }
                    }
                    *(uint4*)(pe) = ev[0];
                    *(uint4*)(pe + 8) = ev[1];
                    *(uint4*)(po) = od[0];
                    *(uint4*)(po + 8) = od[1];
                }
            }

            __syncthreads();              // everyone is done reading plane A
            write_plane((mB + 1) & 1);
            __syncthreads();
        }
        if constexpr (FUSE == 2) {
            // sums over the 32 voxel lanes of each lane half; lane 0 of half h writes cins 16 h .. 16 h + 15 of the tile
#pragma unroll
            for (int i = 0; i < 16; ++i)
#pragma unroll
                for (int off = 16; off > 0; off >>= 1) {
                    st1[i] += __shfl_xor(st1[i], off, 64);
                    st2[i] += __shfl_xor(st2[i], off, 64);
                }
            if (t == 0) G.stat_key[g * G.max_seg + seg_i] = n * G.CiT + cit;
            if ((lane & 31) == 0) {
                float* out = G.stat_part + (((long long)g * G.max_seg + seg_i) * 4 + wave) * 64;
#pragma unroll
                for (int j = 0; j < 16; ++j) {
                    out[16 * (lane >> 5) + j] = st1[j];
                    out[32 + 16 * (lane >> 5) + j] = st2[j];
                }
            }
            ++seg_i;
        }
    }
    if constexpr (FUSE == 2) {
        if (t == 0)
            for (; seg_i < G.max_seg; ++seg_i) G.stat_key[g * G.max_seg + seg_i] = -1;   // unused slots of this workgroup
    }
}

// [Cout][3][3][3][Cin] -> [cin tile][cout chunk][tap][k16][lane][8]: lane (ci = l % 32, half h) holds couts
// chunk * 16 KK + 16 kk + 8 h + j; KK k16-steps per chunk
__global__ void __launch_bounds__(256) dgrad_s2_pack_kernel(const uint16_t* __restrict__ w, uint16_t* __restrict__ wpack, int Cin, int Cout, int KK) {
    const long long total = 27ll * Cin * Cout;
    const long long idx = (long long)blockIdx.x * 256 + threadIdx.x;
    if (idx >= total) return;
    const int j = (int)(idx & 7);
    long long r = idx >> 3;
    const int lane = (int)(r & 63); r >>= 6;
    const int kk = (int)(r % KK); r /= KK;
    const int tap = (int)(r % 27); r /= 27;
    const int nco = Cout / (16 * KK);
    const int chunk = (int)(r % nco);
    const int cit = (int)(r / nco);
    const int ci = cit * 32 + (lane & 31);
    const int co = chunk * 16 * KK + kk * 16 + 8 * (lane >> 5) + j;
    wpack[idx] = w[((long long)co * 27 + tap) * Cin + ci];
}

}  // namespace

static size_t dg2_part_offset(const Geom& g) { return (((size_t)g.w_elems() * 2 + 255) & ~(size_t)255) + 8192; }

bool dgrad_s2_supported(const Geom& g) {
    if (g.dtype != MI3D_BF16 || g.kD != 3 || g.kH != 3 || g.kW != 3) return false;
    if (g.sD != 2 || g.sH != 2 || g.sW != 2) return false;
    if (g.pD != g.pH || g.pD != g.pW || g.pD > 1) return false;
    if (!g.planes_fit_32bit()) return false;
    return g.Cin % 32 == 0 && (g.Cout == 32 || g.Cout % 64 == 0);
}

// the chunked variant applies the optional derivative factor of the geometry while it sums the chunks
bool dgrad_s2_fuses_factor(const Geom& g) { return dgrad_s2_supported(g) && g.Cout > 64; }
bool dgrad_s2_fuses_skip(const Geom& g) { return dgrad_s2_supported(g) && g.Cout >= 64; }
// ... and the unchunked kernel also the sums of the instance-normalisation backward pass of the skip tensor's producer
bool dgrad_s2_fuses_skip_sums(const Geom& g) { return dgrad_s2_supported(g) && g.Cout == 64; }

// workgroups and the most segments (runs along D inside one patch column) one of them walks, for the unchunked kernel
static void dg2_layout(const Geom& g, long long* units, int* nwg, int* max_seg) {
    const int QD = (g.D + 1) / 2, HT = ((g.H + 1) / 2 + RP - 1) / RP, WT = ((g.W + 1) / 2 + CP - 1) / CP;
    *units = (long long)g.N * (g.Cin / 32) * HT * WT * QD;
    int dev = 0, cus = 256;
    if (hipGetDevice(&dev) == hipSuccess) (void)hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev);
    *nwg = (int)(cus < *units ? cus : *units);
    *max_seg = (int)(((*units + *nwg - 1) / *nwg + QD - 1) / QD) + 1;
}

size_t dgrad_s2_workspace_bytes(const Geom& g) {
    if (!dgrad_s2_supported(g)) return 0;
    size_t b = dg2_part_offset(g);   // packed weights + store dump area
    if (g.Cout > 64) b += (size_t)(g.Cout / 64) * g.in_voxels() * g.Cin * sizeof(float);
    if (g.Cout == 64) {   // partial sums and keys of the variant with the normalisation's sums
        long long units; int nwg, max_seg;
        dg2_layout(g, &units, &nwg, &max_seg);
        b += (size_t)nwg * max_seg * (4 * 64 * sizeof(float) + sizeof(int)) + 256;
    }
    return b;
}

int dgrad_s2(const Geom& g, const void* dy, const void* w, void* dx, void* ws, size_t ws_bytes, hipStream_t s) {
    if (ws_bytes < dgrad_s2_workspace_bytes(g)) return MI3D_ERR_WORKSPACE;
    const long long total = g.w_elems();
    const int KK = g.Cout == 32 ? 2 : 4;
    dgrad_s2_pack_kernel<<<(unsigned)((total + 255) / 256), 256, 0, s>>>((const uint16_t*)w, (uint16_t*)ws, g.Cin, g.Cout, KK);
    int st = check_launch();
    if (st) return st;
    Dg2Params G;
    G.dy = (const uint16_t*)dy; G.wpack = (const uint16_t*)ws; G.dx = (uint16_t*)dx;
    G.dump = (uint16_t*)((char*)ws + (((size_t)g.w_elems() * 2 + 255) & ~(size_t)255));
    G.part = (float*)((char*)ws + dg2_part_offset(g));
    G.add = (const uint16_t*)g.add; G.ref = (const uint16_t*)g.ref; G.slope = g.slope;
    // a factor of 1 on both sides of the sign test needs no sign: the store path then reads the added tensor a second
    // time (from the cache) instead of streaming a third tensor of dx's size from memory
    const bool sums = g.add && g.stats;
    if (sums && (!dgrad_s2_fuses_skip_sums(g) || !g.ref || !(g.slope > 0.f))) return MI3D_ERR_UNSUPPORTED;
    if (g.add && g.slope == 1.f) G.ref = G.add;
    if (sums) {   // the factor stays 1; the slope is that of the activation whose inverse enters the sums
        G.ref = (const uint16_t*)g.ref; G.slope = 1.f; G.stat_slope = g.slope;
        long long units; int n2;
        dg2_layout(g, &units, &n2, &G.max_seg);
        G.stat_part = (float*)((char*)ws + dg2_part_offset(g));
        G.stat_key = (int*)(G.stat_part + (size_t)n2 * G.max_seg * 4 * 64);
    }
    G.N = g.N; G.D = g.D; G.H = g.H; G.W = g.W; G.Cin = g.Cin; G.Cout = g.Cout;
    G.Do = g.Do; G.Ho = g.Ho; G.Wo = g.Wo; G.p = g.pD;
    G.QD = (g.D + 1) / 2;
    G.HT = ((g.H + 1) / 2 + RP - 1) / RP;
    G.WT = ((g.W + 1) / 2 + CP - 1) / CP;
    G.CiT = g.Cin / 32;
    G.NCO = g.Cout / (16 * KK);
    G.units = (long long)g.N * G.CiT * G.NCO * G.HT * G.WT * G.QD;
    int dev = 0, cus = 256;
    if (hipGetDevice(&dev) == hipSuccess) (void)hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev);
    const long long nwg = cus < G.units ? cus : G.units;
    G.nwg = (int)nwg;
    const size_t lds = (size_t)27 * KK * 1024 + 2 * (size_t)(2 * KK) * SLABV * 16;
    static std::atomic<bool> attr_set{false};   // set once per process; a second thread racing here repeats an idempotent call
    if (!attr_set) {
        const int max_lds = 27 * 4 * 1024 + 2 * 8 * SLABV * 16;
        const void* fns[10] = {(const void*)dgrad_s2_kernel<0, 2, false>, (const void*)dgrad_s2_kernel<1, 2, false>,
                               (const void*)dgrad_s2_kernel<0, 4, false>, (const void*)dgrad_s2_kernel<1, 4, false>,
                               (const void*)dgrad_s2_kernel<0, 4, true>, (const void*)dgrad_s2_kernel<1, 4, true>,
                               (const void*)dgrad_s2_kernel<0, 4, false, 1>, (const void*)dgrad_s2_kernel<1, 4, false, 1>,
                               (const void*)dgrad_s2_kernel<0, 4, false, 2>, (const void*)dgrad_s2_kernel<1, 4, false, 2>};
        for (const void* f : fns) {
            hipError_t e = hipFuncSetAttribute(f, hipFuncAttributeMaxDynamicSharedMemorySize, max_lds);
            if (e != hipSuccess) { note_hip_error(e); return MI3D_ERR_HIP; }
        }
        attr_set = true;
    }
    const bool part = G.NCO > 1;
    const bool fuse = g.add && !part;    // (Cout == 64: the only unchunked shape with an added gradient)
    if (g.add && !dgrad_s2_fuses_skip(g)) return MI3D_ERR_UNSUPPORTED;
    if (sums) {
        if (g.pD == 0) dgrad_s2_kernel<0, 4, false, 2><<<(unsigned)nwg, 256, lds, s>>>(G);
        else dgrad_s2_kernel<1, 4, false, 2><<<(unsigned)nwg, 256, lds, s>>>(G);
        st = check_launch();
        if (st) return st;
        return sp_stats_finish(G.stat_part, G.stat_key, g.Cin, G.CiT, g.N, G.nwg, G.max_seg, 1.0 / ((double)g.D * g.H * g.W), 0.f, 1, g.stats, s);
    }
    if (fuse && g.pD == 0) dgrad_s2_kernel<0, 4, false, 1><<<(unsigned)nwg, 256, lds, s>>>(G);
    else if (fuse) dgrad_s2_kernel<1, 4, false, 1><<<(unsigned)nwg, 256, lds, s>>>(G);
    else if (part && g.pD == 0) dgrad_s2_kernel<0, 4, true><<<(unsigned)nwg, 256, lds, s>>>(G);
    else if (part) dgrad_s2_kernel<1, 4, true><<<(unsigned)nwg, 256, lds, s>>>(G);
    else if (g.pD == 0 && KK == 2) dgrad_s2_kernel<0, 2, false><<<(unsigned)nwg, 256, lds, s>>>(G);
    else if (g.pD == 0) dgrad_s2_kernel<0, 4, false><<<(unsigned)nwg, 256, lds, s>>>(G);
    else if (KK == 2) dgrad_s2_kernel<1, 2, false><<<(unsigned)nwg, 256, lds, s>>>(G);
    else dgrad_s2_kernel<1, 4, false><<<(unsigned)nwg, 256, lds, s>>>(G);
    st = check_launch();
    if (st || !part) return st;
    const long long n = (long long)g.in_voxels() * g.Cin;
    long long blocks = (n / 8 + 255) / 256;
    if (blocks > 8192) blocks = 8192;
    sum_chunks_bf16_kernel<<<(unsigned)blocks, 256, 0, s>>>(G.part, (uint16_t*)dx, n / 8, n, G.NCO, g.slope, (const uint16_t*)g.ref, nullptr, 0,
                                                            (const uint16_t*)g.add);
    return check_launch();
}

}  // namespace mi3d
