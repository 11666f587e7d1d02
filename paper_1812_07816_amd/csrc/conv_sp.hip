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
#include <type_traits>

#include "mi3d_internal.h"

// The file is compiled twice: as it is (16-row patches, 4 rows per wave, namespace th16) and from conv_sp12.hip with
// 12-row patches of 3 rows per wave (namespace th12) for planes whose height 16-row patches cover badly (24 and 12
// rows: a quarter of the MFMA work would fall on rows outside the tensor).  The entry points at the end of the
// 16-row build choose between the two.
#ifndef SP_TH
#define SP_TH 16
#define SP_RH 4
#define SP_NS th16
#endif

namespace mi3d {
namespace SP_NS {
namespace {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;

constexpr int TH = SP_TH, TW = 32, RH = SP_RH;     // output patch per workgroup, rows per wave
// Waves and threads per workgroup.  RH = 2 gives eight waves, two per SIMD, so that one wave's LDS reads, conversions
// and waits run in the shadow of the other's MFMAs (the counters show that a wave issues nothing else while its own
// MFMA runs).  Measured: 9 % fewer cycles for the 32-channel kernel and the same run time (that kernel is limited by
// power, the clock drops by as much), and register spills in the 64-channel and streamed-weight variants, which need
// about 280 registers against the 256 a wave has with two per SIMD: four waves of four rows it stays.
constexpr int NW = TH / RH, NT = 64 * NW;
// PAIRED (12-row build): where the last column of patches has at most 16 columns inside the tensor (W = 48: 32 + 16),
// a workgroup takes that column for two patch rows at once: MFMA columns 0..15 are the 16 columns of patch row 2 i,
// columns 16..31 the same 16 columns of patch row 2 i + 1, so no MFMA column is spent outside the tensor.  The two
// input patches (18 columns each with halo) sit side by side in the staged rows.
constexpr bool PAIRED = TH == 12;
constexpr int HALF = TW / 2 + 2;                   // staged columns of one half of a paired patch
constexpr int IN_ROWS = TH + 2, IN_COLS = PAIRED ? 2 * HALF : TW + 2;  // with halo
constexpr int COLS = IN_COLS + 1;                  // padded row pitch (voxels) in LDS
constexpr int NLOAD = (IN_ROWS * COLS + 64 * (NW / 4) - 1) / (64 * (NW / 4));   // 16-byte loads per thread per plane (10)
// 16-byte positions per 8-channel slab: IN_ROWS x 35 used (630), room for NLOAD 64-position loads per slab (640),
// slab pitch = 96 bytes mod 256 (646 positions)
constexpr int NV = ((64 * NLOAD * (NW / 4) + 15) / 16) * 16 + 6;
constexpr int STAGE_BYTES = 4 * NV * 16;           // 4 slabs of 8 channels, 16 B per voxel
constexpr int W_BYTES = 27 * 2 * 64 * 16;          // 27 taps x 2 k16 steps x 1 KB fragments
static_assert(NW % 4 == 0 && NLOAD * NW * 16 >= IN_ROWS * IN_COLS && (NV * 16) % 256 == 96, "staging plan");
constexpr unsigned OOB = 0x80000000u;              // buffer offset of a piece that must read as zero

struct SpParams {
    const uint16_t* x;
    const uint16_t* wpack;  // [cout tile][cin chunk][kw][kd][kh][k16][lane][8]
    uint16_t* y;
    uint16_t* dump;         // 8 KB that masked store lanes write to instead of y
    float* part;            // [cin chunk][voxel][Cout] fp32 partial outputs (chunked variant)
    int NCH;                // cin chunks of the chunked variant
    float slope;            // LeakyReLU slope applied to the output (1 = none); with ref: the factor where ref <= 0
    const uint16_t* ref;    // MASK variant: tensor of the output's shape whose sign selects the factor 1 or slope
    int N, D, H, W, Cin, Cout, Do, Ho, Wo, pD, pH, pW;
    int HT, WT, CT;         // tiles per plane, cout tiles
    int WTF, HTP;           // columns of patches taken one patch at a time, paired patch rows of the last column (else 0)
    // Tensors given as two halves along the channels (virtual concatenation): chunks >= xsplit of the input come
    // from x2, cout tiles >= ysplit of the output go to y2; xpitch / ypitch are the channels per voxel of the
    // tensors in memory (Cin, Cout when not split; then the split indices lie beyond the last chunk / tile).
    const uint16_t* x2;
    uint16_t* y2;
    int xpitch, ypitch, xsplit, ysplit;
    float stat_slope;       // STATS = 2: slope of the LeakyReLU whose derivative and inverse enter the sums
    // STATS variants: per-(workgroup, segment, wave) sums of two quantities over the voxels, 32 couts each:
    // [logical workgroup][segment of its unit range][wave][sum, sum of squares][32 couts]
    float* stat_part;
    int* stat_key;          // [logical workgroup][segment]: sample * CT + cout tile of the partial, -1 = unused
    int max_seg;
    long long units;        // N*CT*HT*WT*Do
    int nwg;
};

__device__ __forceinline__ f32x16 mfma(bf16x8 a, bf16x8 b, f32x16 c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}

typedef __attribute__((__vector_size__(2 * sizeof(float)))) float f32x2;
typedef __attribute__((__vector_size__(2 * sizeof(__bf16)))) __bf16 bf16x2;

// Register fragments.  x: input rows row0 .. row0+RH+1 at one (kw, k16)
// position (double buffered); w: the 3 kh taps of one kd group.
struct XFrag { bf16x8 v[RH + 2]; };
struct WFrag { bf16x8 v[3]; };

template <int SUB>
__device__ __forceinline__ void load_x(XFrag& f, const char* in_lane) {
    constexpr int kw = SUB / 2, kk = SUB % 2;
#pragma unroll
    for (int r = 0; r < RH + 2; ++r) f.v[r] = *(const bf16x8*)(in_lane + (2 * kk * NV + r * COLS + kw) * 16);
}
template <int SUB, int KD>
__device__ __forceinline__ void load_w(WFrag& f, const char* w_lane) {
    constexpr int kw = SUB / 2, kk = SUB % 2;
#pragma unroll
    for (int kh = 0; kh < 3; ++kh) f.v[kh] = *(const bf16x8*)(w_lane + (((kw * 3 + KD) * 3 + kh) * 2 + kk) * 1024);
}

// The 12 MFMAs of one kd group at one (kw, k16) position.  The accumulator
// set of output plane od = j - kd is (PH - kd) mod 3.  The kd = 0 set starts a
// new output plane: its first contribution (SUB 0, kh 0) accumulates onto zero.
template <int PH, int SUB, int KD, bool ZERO>
__device__ __forceinline__ void group_mfma(f32x16 (&acc)[3][RH], const XFrag& x, const WFrag& w) {
#pragma unroll
    for (int kh = 0; kh < 3; ++kh) {
#pragma unroll
        for (int r = 0; r < RH; ++r) {
            f32x16& a = acc[(PH + 3 - KD) % 3][r];
            if (ZERO && KD == 0 && SUB == 0 && kh == 0) {
                f32x16 z = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
                a = mfma(w.v[kh], x.v[r + kh], z);
            } else {
                a = mfma(w.v[kh], x.v[r + kh], a);
            }
        }
    }
}

__device__ __forceinline__ void convert_rows(const f32x16 (&a)[RH], uint32_t (&o)[RH][8], float slope);
__device__ __forceinline__ void convert_rows(const f32x16 (&a)[RH], float (&o)[RH][16], float slope);

#define SP_FENCE() __builtin_amdgcn_sched_barrier(0)

// One (kw, k16) position: kd groups 2, 1, 0 (oldest output plane first), with
// the LDS reads of the next position issued between the groups so that they
// are in flight for at least one group of MFMAs.
template <int PH, int SUB, bool ZERO, bool LAST, class Out, class Hook>
__device__ __forceinline__ void sub_step(f32x16 (&acc)[3][RH], XFrag& xc, XFrag& xn, WFrag& w2, WFrag& w1, WFrag& w0,
                                         const char* in_lane, const char* w_lane, Out& outp, float slope, int kdmask, Hook&& hook) {
    constexpr bool last = SUB == 5;
    load_w<SUB, 0>(w0, w_lane);
    if (kdmask & 4) group_mfma<PH, SUB, 2, ZERO>(acc, xc, w2);
    hook(3 * SUB + 0);
    SP_FENCE();
    if (!last) load_x<last ? 0 : SUB + 1>(xn, in_lane);
    if (last && LAST) convert_rows(acc[(PH + 1) % 3], outp, slope);
    if (kdmask & 2) group_mfma<PH, SUB, 1, ZERO>(acc, xc, w1);
    hook(3 * SUB + 1);
    SP_FENCE();
    if (!last) load_w<last ? 0 : SUB + 1, 2>(w2, w_lane);
    if (kdmask & 1) group_mfma<PH, SUB, 0, ZERO>(acc, xc, w0);
    hook(3 * SUB + 2);
    SP_FENCE();
    if (!last) load_w<last ? 0 : SUB + 1, 1>(w1, w_lane);
}

// The MFMAs of one staged input plane.  kdmask bit kd: output plane j - kd lies
// inside the segment; the groups of the other taps are skipped (first and last
// two steps of a segment), so no MFMA work is wasted on planes nobody stores.
// hook(k), k = 0..17, is called once per group of 12 MFMAs: the caller spreads
// its global loads and stores over the step with it, so that no wave ever
// queues a burst of vector-memory instructions.
// ZERO: this stage is the first input-channel chunk of its plane (the new
// output plane starts from zero); LAST: it is the last chunk (the oldest
// output plane is complete and is converted to bf16).
// phase_end(k), k = 0, 1, is called after the two positions of kw = k (the streamed-weight kernel refills
// a weight slot and synchronises there).
template <int PH, bool ZERO, bool LAST, class Out, class Hook, class PhaseEnd>
__device__ __forceinline__ void plane_compute(f32x16 (&acc)[3][RH], const char* in_lane, const char* w_lane,
                                              Out& outp, float slope, int kdmask, Hook&& hook, PhaseEnd&& phase_end) {
    XFrag xa, xb;
    WFrag w2, w1, w0;
    load_x<0>(xa, in_lane);
    load_w<0, 2>(w2, w_lane);
    load_w<0, 1>(w1, w_lane);
    sub_step<PH, 0, ZERO, LAST>(acc, xa, xb, w2, w1, w0, in_lane, w_lane, outp, slope, kdmask, hook);
    sub_step<PH, 1, ZERO, LAST>(acc, xb, xa, w2, w1, w0, in_lane, w_lane, outp, slope, kdmask, hook);
    phase_end(0);
    sub_step<PH, 2, ZERO, LAST>(acc, xa, xb, w2, w1, w0, in_lane, w_lane, outp, slope, kdmask, hook);
    sub_step<PH, 3, ZERO, LAST>(acc, xb, xa, w2, w1, w0, in_lane, w_lane, outp, slope, kdmask, hook);
    phase_end(1);
    sub_step<PH, 4, ZERO, LAST>(acc, xa, xb, w2, w1, w0, in_lane, w_lane, outp, slope, kdmask, hook);
    sub_step<PH, 5, ZERO, LAST>(acc, xb, xa, w2, w1, w0, in_lane, w_lane, outp, slope, kdmask, hook);
}

// fp32 accumulators of one finished output plane -> LeakyReLU (max(v, slope v), 0 <= slope <= 1) -> packed bf16 (RNE)
__device__ __forceinline__ void convert_rows(const f32x16 (&a)[RH], uint32_t (&o)[RH][8], float slope) {
#pragma unroll
    for (int r = 0; r < RH; ++r)
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            f32x2 v = {fmaxf(a[r][2 * i], slope * a[r][2 * i]), fmaxf(a[r][2 * i + 1], slope * a[r][2 * i + 1])};
            bf16x2 b = __builtin_convertvector(v, bf16x2);
            o[r][i] = __builtin_bit_cast(uint32_t, b);
        }
}

// chunked variant: the fp32 accumulators are kept as they are (the activation follows the sum of the chunks)
__device__ __forceinline__ void convert_rows(const f32x16 (&a)[RH], float (&o)[RH][16], float) {
#pragma unroll
    for (int r = 0; r < RH; ++r)
#pragma unroll
        for (int i = 0; i < 16; ++i) o[r][i] = a[r][i];
}

// fp32 partial row: accumulator register i of lane (voxel n, half h) is cout 8 (i / 4) + 4 h + i % 4
__device__ __forceinline__ void store_row(const float (&o)[16], float* p, bool ok, float* dump) {
    float* q = ok ? p : dump;
#pragma unroll
    for (int g4 = 0; g4 < 4; ++g4) *(float4*)(q + 8 * g4) = float4{o[4 * g4], o[4 * g4 + 1], o[4 * g4 + 2], o[4 * g4 + 3]};
}

// Lanes l and l+32 hold the two interleaved halves of a voxel's 32 couts
// (4 couts of every group of 8).  Swapping between the lane halves gives each
// lane 16 consecutive couts, stored as two 16-byte pieces.
// Two packed bf16 values times the factor chosen by the sign of the two bf16 values of m (> 0: 1, else slope);
// fp32 product, rounded to nearest even.  A factor of 1 returns the input bits.
__device__ __forceinline__ uint32_t scale_pair(uint32_t v, uint32_t m, float slope) {
    float lo = __builtin_bit_cast(float, v << 16), hi = __builtin_bit_cast(float, v & 0xffff0000u);
    lo = (int)(m << 16) > 0 ? lo : lo * slope;
    hi = (int)(m & 0xffff0000u) > 0 ? hi : hi * slope;
    f32x2 f = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(f, bf16x2));
}

// BSUM: the lane also adds, for each of its 16 consecutive couts, g = v * lrelu'(a) to s1 and g * xhat to s2, where v
// is the stored bf16 value, a the value of m at the same place and xhat = a > 0 ? a : a / slope (the inverse of the
// LeakyReLU); lanes with nothing to store add zeros.
template <bool MASK, bool BSUM = false>
__device__ __forceinline__ void store_row(const uint32_t (&o)[8], uint16_t* p, bool ok, uint16_t* dump, const uint4 (&m)[2], float slope,
                                          float* s1 = nullptr, float* s2 = nullptr, float bslope = 1.f, bool sum = false) {
    typedef __attribute__((ext_vector_type(2))) unsigned u32x2;
    uint4 c[2];
#pragma unroll
    for (int k = 0; k < 2; ++k) {  // k = 0: cout groups 0 and 2, k = 1: groups 1 and 3
        u32x2 s0 = __builtin_amdgcn_permlane32_swap(o[2 * k], o[2 * k + 4], false, false);
        u32x2 s1_ = __builtin_amdgcn_permlane32_swap(o[2 * k + 1], o[2 * k + 5], false, false);
        c[k].x = s0[0]; c[k].y = s1_[0]; c[k].z = s0[1]; c[k].w = s1_[1];
        if (MASK) {
            c[k].x = scale_pair(c[k].x, m[k].x, slope); c[k].y = scale_pair(c[k].y, m[k].y, slope);
            c[k].z = scale_pair(c[k].z, m[k].z, slope); c[k].w = scale_pair(c[k].w, m[k].w, slope);
        }
    }
    if (BSUM && sum) {   // (uniform)
        const uint32_t cw[8] = {c[0].x, c[0].y, c[0].z, c[0].w, c[1].x, c[1].y, c[1].z, c[1].w};
        const uint32_t mw[8] = {m[0].x, m[0].y, m[0].z, m[0].w, m[1].x, m[1].y, m[1].z, m[1].w};
        const float inv = 1.f / bslope;
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const uint32_t v = ok ? cw[i] : 0u, a = ok ? mw[i] : 0u;
            const float vlo = __builtin_bit_cast(float, v << 16), vhi = __builtin_bit_cast(float, v & 0xffff0000u);
            const float alo = __builtin_bit_cast(float, a << 16), ahi = __builtin_bit_cast(float, a & 0xffff0000u);
            const float glo = alo > 0.f ? vlo : bslope * vlo, ghi = ahi > 0.f ? vhi : bslope * vhi;
            const float xlo = alo > 0.f ? alo : alo * inv, xhi = ahi > 0.f ? ahi : ahi * inv;
            s1[2 * i] += glo; s2[2 * i] = fmaf(glo, xlo, s2[2 * i]);
            s1[2 * i + 1] += ghi; s2[2 * i + 1] = fmaf(ghi, xhi, s2[2 * i + 1]);
        }
    }
    // Unconditional stores: lanes outside the tensor (or with nothing pending) write to the dump area.
    // Behind a branch the compiler cannot count the stores in its vmcnt bookkeeping and makes the next
    // stage's LDS write wait for vmcnt(0), i.e. for these stores to complete.
    uint16_t* q = ok ? p : dump;
    *(uint4*)q = c[0];
    *(uint4*)(q + 8) = c[1];
}

// NC = input-channel chunks of 32 (Cin = 32 NC).  NC = 1 and 2: all weight
// chunks of the cout tile stay in LDS; NC = 1 double-buffers the staged plane,
// NC = 2 has room for one stage only and takes a second barrier per stage.
// NC = 0: any number of chunks, weights streamed.  LDS holds the weights of
// ONE chunk as three slots (one per kw, 18 KB each); while the positions of
// kw = k are computed, the slot of kw = k + 2 (mod 3) is refilled from L2 with
// the block it needs next, two phases ahead of its use, at the price of a
// barrier per phase and 54 KB of extra L2 traffic per stage.
// PART (with NC = 1): the 32-channel chunks of Cin are separate work units whose weights (54 KB) stay resident; each
// writes fp32 partial outputs and a second kernel adds the chunks in index order.  For the deep, small layers this is
// two to three times faster than streaming the weights of all chunks through LDS for every staged plane.
// STATS = 1 (forward, not with PART or MASK): the kernel also adds up y and y^2 per output channel (of the bf16 values it
// stores) for the instance normalisation that follows the convolution (Section 4.1).  Every lane keeps the sums of its
// 16 couts over the rows and planes of a segment; at the end of the segment they are added over the 32 voxel lanes in
// a fixed butterfly and written as one partial per (workgroup, segment, wave).  A second kernel adds the partials of a
// (sample, channel) in index order in double.
// STATS = 2 (data gradient, not with PART or MASK): the same machinery adds up the two sums the backward pass of the
// instance normalisation of the layer below needs: with a = P.ref (that layer's activated output), g = dx * lrelu'(a)
// and xhat = lrelu^-1(a), the sums of g and of g * xhat per channel.  dx itself is stored unchanged.
// MASK (data gradient, not with PART): every output element is multiplied by 1 where P.ref is > 0 and by P.slope
// elsewhere (LeakyReLU derivative of the layer below) after its rounding to bf16 and rounded again: the bits of the
// plain kernel followed by an elementwise pass, without that pass's read and write of the gradient.
template <int NC, bool PART = false, bool MASK = false, int STATS = 0>
__global__ void __launch_bounds__(NT, NW / 4) sp_conv_kernel(SpParams P) {
    extern __shared__ __attribute__((aligned(16))) char lds[];
    constexpr bool STREAM = NC == 0;
    constexpr bool REF = MASK || STATS == 2;   // the kernel reads P.ref at the store addresses
    constexpr int NBUF = NC == 2 ? 1 : 2;
    const int nc = STREAM ? P.Cin / 32 : NC;
    char* w_lds = lds;
    char* in_lds = lds + (STREAM ? 1 : NC) * W_BYTES;
    constexpr int WSLOT = W_BYTES / 3, WPIECES = WSLOT / 16, NWL = (WPIECES + NT - 1) / NT;  // 18 KB, 1152 pieces

    const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
    // XCD-aware placement: hardware deals consecutive workgroup ids round-robin
    // over the 8 XCDs; give each XCD one contiguous range of units so that
    // neighbouring patches (which share halos) meet in the same L2.
    int g = blockIdx.x;
    if ((P.nwg & 7) == 0) g = (g & 7) * (P.nwg >> 3) + (g >> 3);
    long long u0 = P.units * g / P.nwg, u1 = P.units * (g + 1) / P.nwg;

    // Staging (double-buffered variants): wave w fills slab w (channels 8w..8w+7 of the chunk) of the next
    // stage with ten direct-to-LDS buffer loads; load i covers the 64 LDS positions 64 i .. 64 i + 63 of the
    // slab (position = row * 35 + col), lane l position 64 i + l.  The data never passes through registers:
    // no ds_write, no wait before it (the LDS write phase at the end of a stage cost about 900 cycles of
    // 9400), and zero padding comes from the buffer's range check (offset OOB reads as 0).  The NC = 2
    // variant has one stage buffer only and keeps the register path: piece i of a thread there is channels
    // 8c..8c+7, c = l / 16, of voxel 16 (4 i + w) + l % 16 of the patch, row-major over 18 x 34.
    constexpr bool DMA = NC != 2;
    constexpr int NVOX = IN_ROWS * IN_COLS;
    const int wave_u = __builtin_amdgcn_readfirstlane(wave);
    int lds_off[DMA ? 1 : NLOAD];
    if (!DMA) {
#pragma unroll
        for (int i = 0; i < NLOAD; ++i) {
            int v = 16 * (NW * i + wave) + (lane & 15), c = lane >> 4;
            int row = v / IN_COLS, col = v - row * IN_COLS;
            lds_off[i] = (c * NV + row * COLS + col) * 16;
        }
    }
    f32x16 acc[3][RH];
    const char* w_lane = w_lds + lane * 16;

    int cur_ct = -1;
    int seg = 0;   // STATS: index of the segment within this workgroup's unit range
    while (u0 < u1) {
        long long column = u0 / P.Do;
        int od_start = (int)(u0 - column * P.Do);
        int od_end = od_start + (int)((u1 - u0) < (long long)(P.Do - od_start) ? (u1 - u0) : (long long)(P.Do - od_start));
        u0 += od_end - od_start;
        const int tpp = P.HT * P.WTF + P.HTP;                  // patches of a plane
        const int tsel = (int)(column % tpp); column /= tpp;
        const bool paired = PAIRED && tsel >= P.HT * P.WTF;    // (uniform)
        const int wtf1 = P.WTF > 0 ? P.WTF : 1;                // (no unpaired column: every patch is paired)
        const int wt = paired ? P.WTF : tsel % wtf1;
        const int ht = paired ? 2 * (tsel - P.HT * P.WTF) : tsel / wtf1;
        // this lane's column of the patch (before the tap shift) in the staged rows, the rows between its patch and the
        // first one, and its column in the tensor
        const int lcol = paired ? (lane & 15) + ((lane & 16) ? HALF : 0) : (lane & 31);
        const int lrow = paired && (lane & 16) ? TH : 0;
        const int lane_in_off = ((lane >> 5) * NV + wave * RH * COLS + lcol) * 16;
        const int chunk0 = PART ? (int)(column % P.NCH) : 0;   // chunked variant: this unit's cin chunk
        if (PART) column /= P.NCH;
        int ct = (int)(column % P.CT);
        int n = (int)(column / P.CT);
        const int h0 = ht * TH, w0 = wt * TW;

        // packed weights of this cout tile (chunked variant: of this cin chunk of it)
        const char* wct = (const char*)P.wpack + ((long long)ct * (PART ? P.NCH : nc) + chunk0) * W_BYTES;
        if (STREAM) {  // slots kw = 0, 1 of chunk 0; slot 2 follows during the first phase
            for (int i = t; i < 2 * WPIECES; i += NT) ((uint4*)w_lds)[i] = ((const uint4*)wct)[i];
        } else if (ct * (PART ? P.NCH : 1) + chunk0 != cur_ct) {  // (re)load the weights; previous readers passed a barrier
            for (int i = t; i < NC * W_BYTES / 16; i += NT) ((uint4*)w_lds)[i] = ((const uint4*)wct)[i];
            cur_ct = ct * (PART ? P.NCH : 1) + chunk0;
        }
        // (vector type and no pointer table: with a struct type or an indexed table of sources the pieces were kept
        // in scratch memory, whose loads and stores share the counter of the global loads)
        typedef __attribute__((ext_vector_type(4))) unsigned u32x4;
        u32x4 wreg[NWL];
        const int wlast = t + NT * (NWL - 1) < WPIECES ? t + NT * (NWL - 1) : WPIECES - 1;
        auto write_wslot = [&](int slot) {
#pragma unroll
            for (int i = 0; i < NWL; ++i)
                if (t + NT * i < WPIECES) *(u32x4*)(w_lds + slot * WSLOT + (t + NT * i) * 16) = wreg[i];
        };
        // offsets of this thread's pieces relative to the plane base: bytes (DMA) or elements (register path)
        int goff[NLOAD];
        unsigned valid = 0;
#pragma unroll
        for (int i = 0; i < NLOAD; ++i) {
            int row, col, c;
            bool ok;
            if (DMA) {
                const int pos = 64 * (i + NLOAD * (wave >> 2)) + lane;   // the NW / 4 waves of a slab share its ten loads
                row = pos / COLS; col = pos - row * COLS;
                c = wave & 3;
                ok = row < IN_ROWS && col < (paired ? IN_COLS : TW + 2);
            } else {
                const int v = 16 * (NW * i + wave) + (lane & 15);
                row = v / IN_COLS; col = v - row * IN_COLS;
                c = lane >> 4;
                ok = v < NVOX && col < (paired ? IN_COLS : TW + 2);
            }
            const bool second = paired && col >= HALF;   // the patch one patch row further down
            const int gh = h0 + (second ? TH : 0) - P.pH + row, gw = w0 - P.pW + (second ? col - HALF : col);
            ok = ok && gh >= 0 && gh < P.H && gw >= 0 && gw < P.W;
            if (DMA) goff[i] = ok ? ((gh * P.W + gw) * P.xpitch + c * 8) * 2 : (int)OOB;
            else goff[i] = ok ? (gh * P.W + gw) * P.xpitch + c * 8 : 0;
            valid |= (ok ? 1u : 0u) << i;
        }
        const long long plane_elems = (long long)P.H * P.W * P.xpitch;
        const uint16_t* xn = P.x + (long long)n * P.D * plane_elems;
        const uint16_t* xn2 = P.x2 + (long long)n * P.D * plane_elems;
        const int ct_local = ct >= P.ysplit ? ct - P.ysplit : ct;
        uint16_t* yn = (ct >= P.ysplit ? P.y2 : P.y) + (long long)n * P.Do * P.Ho * P.Wo * P.ypitch;
        const int opitch = PART ? P.Cout : P.ypitch;   // the fp32 partial outputs are dense
        const int nJ = od_end - od_start + 2;
        uint4 pre[DMA ? 1 : NLOAD];

        // A plane outside [0, D) is zero padding.  DMA: its buffer has zero records, so every piece reads 0.
        // Register path: loads are unconditional (masked pieces read element 0 of a valid plane) and zeroed
        // afterwards, so that the piece registers never pass through memory.
        unsigned pre_mask = 0;
        const uint16_t* pre_base = xn;
        __amdgpu_buffer_rsrc_t rsrc = __builtin_amdgcn_make_buffer_rsrc((void*)xn, 0, 0, 0x00020000);
        auto begin_stage = [&](int ip, int chunk) {
            const bool inside = ip >= 0 && ip < P.D;
            chunk += chunk0;
            const bool high = chunk >= P.xsplit;
            if (high) chunk -= P.xsplit;
            pre_base = (high ? xn2 : xn) + (long long)(inside ? ip : 0) * plane_elems + chunk * 32;
            pre_mask = inside ? valid : 0u;
            if (DMA) rsrc = __builtin_amdgcn_make_buffer_rsrc((void*)pre_base, 0, inside ? (int)(plane_elems * 2) - chunk * 64 : 0, 0x00020000);
        };
        // DMA: piece i of the stage begun last goes to stage buffer buf
        auto load_piece = [&](int i, int buf) {
            if (DMA) {
                typedef __attribute__((address_space(3))) void* lds_ptr;
                __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc, (lds_ptr)(in_lds + buf * STAGE_BYTES + ((wave_u & 3) * NV + 64 * (i + NLOAD * (wave_u >> 2))) * 16), 16, goff[i], 0, 0, 0);
            } else {
                pre[i] = *(const uint4*)(pre_base + goff[i]);
            }
        };
        // register path only; the zeroing of masked pieces happens here, after the MFMA work, so
        // that nothing waits for the global loads before the compute starts
        auto write_stage = [&](int buf) {
            if (DMA) return;
            char* dst = in_lds + buf * STAGE_BYTES;
#pragma unroll
            for (int i = 0; i < NLOAD; ++i) {
                const bool ok = (pre_mask >> i) & 1;
                uint4 v;
                v.x = ok ? pre[i].x : 0u;
                v.y = ok ? pre[i].y : 0u;
                v.z = ok ? pre[i].z : 0u;
                v.w = ok ? pre[i].w : 0u;
                if (16 * (NW * i + wave) + (lane & 15) < NVOX) *(uint4*)(dst + lds_off[i]) = v;
            }
        };
        // finished rows wait in outp[] and are stored during the next stage
        typename std::conditional<PART, float[RH][16], uint32_t[RH][8]>::type outp;
        long long st_off = 0;     // element offset of row 0 of the pending plane for this lane (before the lane half)
        float* partn = PART ? P.part + ((long long)chunk0 * P.N + n) * P.Do * P.Ho * P.Wo * P.Cout : nullptr;
        bool st_pending = false;
        const int ow_ = w0 + (paired ? (lane & 15) : (lane & 31));
        const long long row_pitch = (long long)P.Wo * opitch;
        uint4 mk[REF ? RH : 1][2];   // the pieces of ref at the addresses of the pending stores
        const uint16_t* refn = REF ? P.ref + (long long)n * P.Do * P.Ho * P.Wo * P.Cout : nullptr;
        auto load_mask = [&](int r) {     // unconditional, like the stores: masked lanes read the dump area
            if constexpr (REF) {
                const bool ok = st_pending && ow_ < P.Wo && h0 + lrow + wave * RH + r < P.Ho;
                const uint16_t* q = ok ? refn + st_off + r * row_pitch + 16 * (lane >> 5) : P.dump + lane * 16;
                mk[r][0] = *(const uint4*)q;
                mk[r][1] = *(const uint4*)(q + 8);
            }
        };
        float st1[STATS ? 16 : 1], st2[STATS ? 16 : 1];   // STATS: this lane's sums over the segment (its 16 couts)
        if constexpr (STATS) {
#pragma unroll
            for (int i = 0; i < 16; ++i) st1[i] = st2[i] = 0.f;
        }
        auto store_piece = [&](int r) {
            const bool ok = st_pending && ow_ < P.Wo && h0 + lrow + wave * RH + r < P.Ho;
            if (STATS == 1 && st_pending) {   // (uniform: stages with nothing to store skip the arithmetic)
#pragma unroll
                for (int i = 0; i < 8; ++i) {
                    const uint32_t v = ok ? outp[r][i] : 0u;
                    const float lo = __builtin_bit_cast(float, v << 16), hi = __builtin_bit_cast(float, v & 0xffff0000u);
                    st1[2 * i] += lo; st2[2 * i] = fmaf(lo, lo, st2[2 * i]);
                    st1[2 * i + 1] += hi; st2[2 * i + 1] = fmaf(hi, hi, st2[2 * i + 1]);
                }
            }
            if constexpr (PART) store_row(outp[r], partn + st_off + r * row_pitch + 4 * (lane >> 5), ok, (float*)P.dump + lane * 32);
            else store_row<MASK, STATS == 2>(outp[r], yn + st_off + r * row_pitch + 16 * (lane >> 5), ok, P.dump + lane * 16, mk[REF ? r : 0], P.slope,
                                             st1, st2, P.stat_slope, st_pending);
        };

        // every segment starts from cleared accumulators (keeps them dead across segments)
#pragma unroll
        for (int s = 0; s < 3; ++s)
#pragma unroll
            for (int r = 0; r < RH; ++r)
#pragma unroll
                for (int i = 0; i < 16; ++i) acc[s][r][i] = 0.f;

        begin_stage(od_start - P.pD, 0);
#pragma unroll
        for (int i = 0; i < NLOAD; ++i) load_piece(i, 0);
        write_stage(0);
        if (DMA) asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __syncthreads();

        // Plane step jj stages input plane ip = od_start + jj - pD, one 32-channel chunk at a time, and
        // completes output plane od_start + jj - 2.  Hook slots 0..9 issue the loads of the next stage,
        // slots 10..13 the stores of the plane finished last (before slot 15 overwrites outp[]).  Loads and
        // LDS writes are unconditional (after the last stage they fetch a valid plane nobody reads): a
        // condition would hide the load/consumer pairing from the compiler's wait-count insertion.
#define SP_STAGE(PHASE, CHUNK, ZERO, LAST)                                                      \
        {                                                                                       \
            const int j_ = od_start + jj;                                                       \
            const int cnext_ = (CHUNK) + 1 < nc ? (CHUNK) + 1 : 0;                              \
            if ((CHUNK) + 1 < nc) begin_stage(j_ - P.pD, (CHUNK) + 1);                          \
            else begin_stage(j_ + 1 - P.pD, 0);                                                 \
            const int buf_ = NBUF == 2 ? (sq & 1) : 0;                                          \
            /* streamed weights: block refilled during phase k = the next user of slot (k + 2) % 3 */ \
            const char* wsrc0_ = wct + ((CHUNK) * 3 + 2) * WSLOT;                               \
            const char* wsrc1_ = wct + (cnext_ * 3 + 0) * WSLOT;                                \
            const char* wsrc2_ = wct + (cnext_ * 3 + 1) * WSLOT;                                \
            int kdmask_ = 0;                                                                    \
            for (int kd_ = 0; kd_ < 3; ++kd_)                                                   \
                if (jj - kd_ >= 0 && jj - kd_ < nJ - 2) kdmask_ |= 1 << kd_;                    \
            plane_compute<PHASE, ZERO, LAST>(acc, in_lds + buf_ * STAGE_BYTES + lane_in_off,    \
                                             w_lane + (STREAM ? 0 : (CHUNK) * W_BYTES), outp, MASK ? 1.f : P.slope, kdmask_, [&](int k) { \
                if (STREAM && k % 6 == 0) { /* all pieces of the slot at the start of its phase: a full phase of cover */ \
                    const char* ws_ = k / 6 == 0 ? wsrc0_ : k / 6 == 1 ? wsrc1_ : wsrc2_;       \
                    _Pragma("unroll") for (int i_ = 0; i_ < NWL; ++i_) wreg[i_] = *(const u32x4*)(ws_ + (i_ < NWL - 1 ? t + NT * i_ : wlast) * 16); \
                }                                                                               \
                if (k < NLOAD) load_piece(k, NBUF == 2 ? ((sq + 1) & 1) : 0);                   \
                if (REF && k >= NLOAD - RH && k < NLOAD) load_mask(k - (NLOAD - RH));           \
                if (k < NLOAD) {}                                                               \
                else if (k < NLOAD + RH) {                                                      \
                    store_piece(k - NLOAD);                                                     \
                    if (k == NLOAD + RH - 1) st_pending = false;                                \
                }                                                                               \
            }, [&](int k) {                                                                     \
                if (STREAM) { write_wslot((k + 2) % 3); __syncthreads(); }                      \
            });                                                                                 \
            if (STREAM) write_wslot(1);                                                         \
            if (NBUF == 1) __syncthreads(); /* all waves are done reading the only stage */     \
            write_stage(NBUF == 2 ? ((sq + 1) & 1) : 0);                                        \
            if (LAST) {                                                                         \
                st_pending = jj >= 2;                                                           \
                st_off = (((long long)(j_ - 2) * P.Ho + h0 + lrow + wave * RH) * P.Wo + ow_) * opitch + (PART ? ct : ct_local) * 32;  \
            }                                                                                   \
            ++sq;                                                                               \
            /* the loads into the next stage are complete; the 2 RH stores issued after them may still fly */ \
            if (DMA) { if (RH == 4) asm volatile("s_waitcnt vmcnt(8)" ::: "memory"); else if (RH == 3) asm volatile("s_waitcnt vmcnt(6)" ::: "memory"); else asm volatile("s_waitcnt vmcnt(4)" ::: "memory"); } \
            __syncthreads();                                                                    \
        }
#define SP_STEP(PHASE)                                                                          \
        if (NC == 1) { SP_STAGE(PHASE, 0, true, true) }                                         \
        else if (NC == 2) { SP_STAGE(PHASE, 0, true, false) SP_STAGE(PHASE, 1, false, true) }   \
        else {                                                                                  \
            SP_STAGE(PHASE, 0, true, false)                                                     \
            for (int c_ = 1; c_ + 1 < nc; ++c_) SP_STAGE(PHASE, c_, false, false)               \
            SP_STAGE(PHASE, nc - 1, false, true)                                                \
        }
        int sq = 0;  /* stage counter: selects the input buffer */
        for (int jj = 0;;) {
            SP_STEP(0)
            if (++jj >= nJ) break;
            SP_STEP(1)
            if (++jj >= nJ) break;
            SP_STEP(2)
            if (++jj >= nJ) break;
        }
#undef SP_STEP
#undef SP_STAGE
#pragma unroll
        for (int r = 0; r < RH; ++r) load_mask(r);
#pragma unroll
        for (int r = 0; r < RH; ++r) store_piece(r);  // the last plane of the segment
        if constexpr (STATS) {
            // sums over the 32 voxel lanes of each lane half (fixed butterfly), then lane 0 of each half writes its 16
            // couts: accumulator register j of half h is cout 8 (j / 4) + 4 h + j % 4 of the tile (STATS = 1: sums taken
            // before the exchange between the lane halves), cout 16 h + j after it (STATS = 2)
#pragma unroll
            for (int i = 0; i < 16; ++i)
#pragma unroll
                for (int off = 16; off > 0; off >>= 1) {
                    st1[i] += __shfl_xor(st1[i], off, 64);
                    st2[i] += __shfl_xor(st2[i], off, 64);
                }
            if (t == 0) P.stat_key[g * P.max_seg + seg] = n * P.CT + ct;   // whose sums these are
            if ((lane & 31) == 0) {
                float* out = P.stat_part + (((long long)g * P.max_seg + seg) * NW + wave) * 64;
#pragma unroll
                for (int j = 0; j < 16; ++j) {
                    const int c = STATS == 1 ? 8 * (j >> 2) + 4 * (lane >> 5) + (j & 3) : 16 * (lane >> 5) + j;
                    out[c] = st1[j];
                    out[32 + c] = st2[j];
                }
            }
            ++seg;
        }
    }
    if constexpr (STATS) {
        if (t == 0)
            for (; seg < P.max_seg; ++seg) P.stat_key[g * P.max_seg + seg] = -1;   // unused slots of this workgroup
    }
}

// stats[n][c] = (mean, 1 / sqrt(var + eps)) of y over the voxels from the partial sums of the STATS = 1 variant, or
// (means = 1) the plain means of the two sums of the STATS = 2 variant.  A block of 1024 threads per (sample, cout
// tile); thread (slice s of 16, sum q, cout c) adds the partials of every sixteenth workgroup in index order in double
// (key: which (sample, cout tile) a partial belongs to), then the sixteen slices are added in order.
constexpr int FIN_SLICES = 16;
__global__ void __launch_bounds__(64 * FIN_SLICES) sp_stats_finish_kernel(const float* __restrict__ part, const int* __restrict__ key, int Cout, int CT,
                                                                          int nwg, int max_seg, double inv_v, float eps, int means, float* __restrict__ stats) {
    __shared__ double red[FIN_SLICES][64];
    const int t = threadIdx.x, sl = t >> 6, qc = t & 63;     // qc = 32 q + c
    const int mine = blockIdx.x;                             // n * CT + ct
    double a = 0.0;
    for (int g = sl; g < nwg; g += FIN_SLICES)
        for (int seg = 0; seg < max_seg; ++seg)
            if (key[g * max_seg + seg] == mine) {
                const float* p = part + (((long long)g * max_seg + seg) * NW) * 64;
                for (int w = 0; w < NW; ++w) a += (double)p[w * 64 + qc];
            }
    red[sl][qc] = a;
    __syncthreads();
    if (t < 32) {
        double s1 = 0.0, s2 = 0.0;
        for (int k = 0; k < FIN_SLICES; ++k) { s1 += red[k][t]; s2 += red[k][32 + t]; }
        const double mean = s1 * inv_v;
        double var = s2 * inv_v - mean * mean;
        if (var < 0.0) var = 0.0;
        const int n = mine / CT, c = (mine % CT) * 32 + t;
        stats[2 * ((long long)n * Cout + c)] = (float)mean;
        stats[2 * ((long long)n * Cout + c) + 1] = means ? (float)(s2 * inv_v) : (float)(1.0 / sqrt(var + (double)eps));
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

bool supported(const Geom& g, int pass) {
    if (g.dtype != MI3D_BF16 || g.kD != 3 || g.kH != 3 || g.kW != 3) return false;
    if (g.sD != 1 || g.sH != 1 || g.sW != 1) return false;
    if (g.pD > 2 || g.pH > 2 || g.pW > 2) return false;
    // a staged plane is addressed through a buffer resource with 32-bit offsets; 2^31 marks padding
    if ((long long)g.H * g.W * g.Cin * 2 >= (1ll << 31) || (long long)g.Ho * g.Wo * g.Cout * 2 >= (1ll << 31)) return false;
    if (pass == MI3D_PASS_FWD) return g.Cin % 32 == 0 && g.Cout % 32 == 0;
    if (pass == MI3D_PASS_DGRAD) return g.Cout % 32 == 0 && g.Cin % 32 == 0;
    return false;
}

// Patches of an output plane of Ho x Wo: wtf columns of patches are taken one patch at a time; where the last column
// has at most 16 columns inside the tensor and there are at least two patch rows, it is taken two patch rows at a
// time (htp pairs; 12-row build only).
static int sp_plane_tiles(int Ho, int Wo, int* wtf, int* htp) {
    const int HT = (Ho + TH - 1) / TH, WT = (Wo + TW - 1) / TW, tail = Wo - (WT - 1) * TW;
    const bool pair = PAIRED && tail <= TW / 2 && HT >= 2;
    *wtf = pair ? WT - 1 : WT;
    *htp = pair ? (HT + 1) / 2 : 0;
    return HT * *wtf + *htp;
}

static int sp_cu_count() {
    int dev = 0, cus = 256;
    if (hipGetDevice(&dev) == hipSuccess) (void)hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev);
    return cus;
}

// Chunked variant (32-channel chunks of the contracted channels as work units, resident weights, fp32 partial
// outputs): used when the convolution contracts at least 96 channels and has fewer (cout tile, patch, plane) units
// than two per CU, i.e. on the smallest volumes, where whole-Cin units leave most of the chip idle.  Measured at
// N = 1 (chunked / streamed weights): 320->320 at 12^3 0.082 / 0.091 ms, 256->256 at 24^3 0.120 / 0.116,
// 512->256 at 24^3 0.207 / 0.219; with more units the streamed weights win (256->128 at 48^3 0.38 / 0.28).
static bool sp_use_chunks(const Geom& g, int pass) {
    const bool flip = pass == MI3D_PASS_DGRAD;
    const int cin = flip ? g.Cout : g.Cin, cout = flip ? g.Cin : g.Cout;
    const int Do = flip ? g.D : g.Do, Ho = flip ? g.H : g.Ho, Wo = flip ? g.W : g.Wo;
    int wtf, htp;
    const long long units = (long long)g.N * (cout / 32) * sp_plane_tiles(Ho, Wo, &wtf, &htp) * Do;
    return cin >= 96 && units < 2ll * sp_cu_count();
}


static size_t sp_part_offset(const Geom& g) { return (((size_t)g.w_elems() * 2 + 255) & ~(size_t)255) + 8192; }

// STATS variants (unchunked): workgroups, most segments of a workgroup's unit range, bytes of the partial sums
static void sp_stat_layout(const Geom& g, int pass, long long* units, int* nwg, int* max_seg) {
    const bool flip = pass == MI3D_PASS_DGRAD;
    const int cout = flip ? g.Cin : g.Cout, Do = flip ? g.D : g.Do, Ho = flip ? g.H : g.Ho, Wo = flip ? g.W : g.Wo;
    int wtf, htp;
    *units = (long long)g.N * (cout / 32) * sp_plane_tiles(Ho, Wo, &wtf, &htp) * Do;
    long long n = sp_cu_count();
    if (n > *units) n = *units;
    *nwg = (int)n;
    const long long per_wg = (*units + n - 1) / n;
    *max_seg = (int)((per_wg + Do - 1) / Do) + 1;
}
static size_t sp_stat_bytes(const Geom& g, int pass) {
    long long units; int nwg, max_seg;
    sp_stat_layout(g, pass, &units, &nwg, &max_seg);
    return (size_t)nwg * max_seg * (NW * 64 * sizeof(float) + sizeof(int)) + 256;
}
bool fuses_stats(const Geom& g) { return supported(g, MI3D_PASS_FWD) && !sp_use_chunks(g, MI3D_PASS_FWD); }
// the data gradient that also delivers the sums of the instance-normalisation backward pass of the layer below
bool fuses_bwd_sums(const Geom& g) { return supported(g, MI3D_PASS_DGRAD) && !sp_use_chunks(g, MI3D_PASS_DGRAD); }

size_t workspace_bytes(const Geom& g, int pass) {
    if (!supported(g, pass)) return 0;
    size_t b = sp_part_offset(g);  // packed weights + store dump area
    if (sp_use_chunks(g, pass)) {
        const int cin = pass == MI3D_PASS_DGRAD ? g.Cout : g.Cin;
        const size_t out_elems = pass == MI3D_PASS_DGRAD ? (size_t)g.in_voxels() * g.Cin : (size_t)g.out_voxels() * g.Cout;
        b += (size_t)(cin / 32) * out_elems * sizeof(float);
    } else {
        b += sp_stat_bytes(g, pass);   // partial sums of the STATS variants
    }
    return b;
}

// in: activations read (x for fwd, dy for dgrad); out: y or dx
int conv(const Geom& g, int pass, const void* in, const void* w, void* out, void* ws, size_t ws_bytes, hipStream_t s) {
    if (ws_bytes < workspace_bytes(g, pass)) return MI3D_ERR_WORKSPACE;
    const bool flip = pass == MI3D_PASS_DGRAD;
    long long total = g.w_elems();
    sp_pack_weights_kernel<<<(unsigned)((total + 255) / 256), 256, 0, s>>>((const uint16_t*)w, (uint16_t*)ws, g.Cin, g.Cout, flip ? 1 : 0);
    int st = check_launch();
    if (st) return st;
    SpParams P;
    P.x = (const uint16_t*)in;
    P.wpack = (const uint16_t*)ws;
    P.y = (uint16_t*)out;
    P.dump = (uint16_t*)((char*)ws + (((size_t)g.w_elems() * 2 + 255) & ~(size_t)255));
    P.part = (float*)((char*)ws + sp_part_offset(g));
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
    // halves along the channels of the tensor of x's shape: the input of the forward pass, the output of the data gradient
    P.x2 = P.x; P.y2 = P.y; P.xpitch = P.Cin; P.ypitch = P.Cout; P.xsplit = P.Cin; P.ysplit = P.Cout;
    if (g.hi) {
        if (g.Cin % 64) return MI3D_ERR_UNSUPPORTED;
        if (!flip) { P.x2 = (const uint16_t*)g.hi; P.xpitch = g.Cin / 2; P.xsplit = g.Cin / 64; }
        else { P.y2 = (uint16_t*)g.hi; P.ypitch = g.Cin / 2; P.ysplit = g.Cin / 64; }
    }
    const bool chunks = sp_use_chunks(g, pass);
    P.NCH = chunks ? P.Cin / 32 : 1;
    const bool bstat = pass == MI3D_PASS_DGRAD && g.stats;   // sums for the normalisation below; dx itself stays unmasked
    if (bstat && (chunks || !g.ref || g.hi || !(g.slope > 0.f))) return MI3D_ERR_UNSUPPORTED;
    const bool mask = pass == MI3D_PASS_DGRAD && g.ref && g.slope != 1.f && !chunks && !bstat;
    P.slope = (pass == MI3D_PASS_FWD || mask) ? g.slope : 1.f;
    P.ref = mask || bstat ? (const uint16_t*)g.ref : nullptr;
    P.stat_slope = bstat ? g.slope : 1.f;
    P.units = (long long)P.N * P.CT * P.NCH * sp_plane_tiles(P.Ho, P.Wo, &P.WTF, &P.HTP) * P.Do;
    long long nwg = sp_cu_count();
    if (nwg > P.units) nwg = P.units;
    P.nwg = (int)nwg;
    const bool stat = pass == MI3D_PASS_FWD && g.stats;
    if (stat && chunks) return MI3D_ERR_UNSUPPORTED;
    P.stat_part = P.part;   // same place in the workspace as the chunked variant's partial outputs
    P.max_seg = 1;
    P.stat_key = nullptr;
    if (stat || bstat) {
        long long units; int n2;
        sp_stat_layout(g, pass, &units, &n2, &P.max_seg);
        P.stat_key = (int*)(P.stat_part + (size_t)n2 * P.max_seg * NW * 64);
    }
    const int nc = P.Cin / 32;
    const size_t lds1 = W_BYTES + 2 * STAGE_BYTES, lds2 = 2 * W_BYTES + STAGE_BYTES;
    static std::atomic<bool> attr_set{false};   // set once per process; a second thread racing here repeats an idempotent call
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute((const void*)sp_conv_kernel<1>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds1);
        if (e == hipSuccess) e = hipFuncSetAttribute((const void*)sp_conv_kernel<2>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds2);
        if (e == hipSuccess) e = hipFuncSetAttribute((const void*)sp_conv_kernel<0>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds1);
        if (e == hipSuccess) e = hipFuncSetAttribute((const void*)sp_conv_kernel<1, true>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds1);
        if (e == hipSuccess) e = hipFuncSetAttribute((const void*)sp_conv_kernel<1, false, true>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds1);
        if (e == hipSuccess) e = hipFuncSetAttribute((const void*)sp_conv_kernel<2, false, true>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds2);
        if (e == hipSuccess) e = hipFuncSetAttribute((const void*)sp_conv_kernel<0, false, true>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds1);
        if (e == hipSuccess) e = hipFuncSetAttribute((const void*)sp_conv_kernel<1, false, false, 1>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds1);
        if (e == hipSuccess) e = hipFuncSetAttribute((const void*)sp_conv_kernel<2, false, false, 1>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds2);
        if (e == hipSuccess) e = hipFuncSetAttribute((const void*)sp_conv_kernel<0, false, false, 1>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds1);
        if (e == hipSuccess) e = hipFuncSetAttribute((const void*)sp_conv_kernel<1, false, false, 2>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds1);
        if (e == hipSuccess) e = hipFuncSetAttribute((const void*)sp_conv_kernel<2, false, false, 2>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds2);
        if (e == hipSuccess) e = hipFuncSetAttribute((const void*)sp_conv_kernel<0, false, false, 2>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds1);
        if (e != hipSuccess) { note_hip_error(e); return MI3D_ERR_HIP; }
        attr_set = true;
    }
    if (chunks) {
        sp_conv_kernel<1, true><<<(unsigned)nwg, NT, lds1, s>>>(P);
        st = check_launch();
        if (st) return st;
        const long long n = (long long)P.N * P.Do * P.Ho * P.Wo * P.Cout;   // a multiple of 32
        long long blocks = (n / 8 + 255) / 256;
        if (blocks > 8192) blocks = 8192;
        sum_chunks_bf16_kernel<<<(unsigned)blocks, 256, 0, s>>>(P.part, (uint16_t*)out, n / 8, n, P.NCH, g.slope, pass == MI3D_PASS_DGRAD ? (const uint16_t*)g.ref : nullptr,
                                                                flip && g.hi ? (uint16_t*)g.hi : nullptr, P.Cout, nullptr);
        return check_launch();
    }
    if (stat || bstat) {
        if (stat && nc == 1) sp_conv_kernel<1, false, false, 1><<<(unsigned)nwg, NT, lds1, s>>>(P);
        else if (stat && nc == 2) sp_conv_kernel<2, false, false, 1><<<(unsigned)nwg, NT, lds2, s>>>(P);
        else if (stat) sp_conv_kernel<0, false, false, 1><<<(unsigned)nwg, NT, lds1, s>>>(P);
        else if (nc == 1) sp_conv_kernel<1, false, false, 2><<<(unsigned)nwg, NT, lds1, s>>>(P);
        else if (nc == 2) sp_conv_kernel<2, false, false, 2><<<(unsigned)nwg, NT, lds2, s>>>(P);
        else sp_conv_kernel<0, false, false, 2><<<(unsigned)nwg, NT, lds1, s>>>(P);
        st = check_launch();
        if (st) return st;
        sp_stats_finish_kernel<<<P.N * P.CT, 64 * FIN_SLICES, 0, s>>>(P.stat_part, P.stat_key, P.Cout, P.CT, P.nwg, P.max_seg,
                                                          1.0 / ((double)P.Do * P.Ho * P.Wo), g.stats_eps, bstat ? 1 : 0, g.stats);
        return check_launch();
    }
    if (mask && nc == 1) sp_conv_kernel<1, false, true><<<(unsigned)nwg, NT, lds1, s>>>(P);
    else if (mask && nc == 2) sp_conv_kernel<2, false, true><<<(unsigned)nwg, NT, lds2, s>>>(P);
    else if (mask) sp_conv_kernel<0, false, true><<<(unsigned)nwg, NT, lds1, s>>>(P);
    else if (nc == 1) sp_conv_kernel<1><<<(unsigned)nwg, NT, lds1, s>>>(P);
    else if (nc == 2) sp_conv_kernel<2><<<(unsigned)nwg, NT, lds2, s>>>(P);
    else sp_conv_kernel<0><<<(unsigned)nwg, NT, lds1, s>>>(P);
    return check_launch();
}

}  // namespace SP_NS

#if SP_TH == 16
namespace th12 {
size_t workspace_bytes(const Geom& g, int pass);
int conv(const Geom& g, int pass, const void* in, const void* w, void* out, void* ws, size_t ws_bytes, hipStream_t s);
bool fuses_stats(const Geom& g);
bool fuses_bwd_sums(const Geom& g);
}  // namespace th12

// 12-row patches where they cover the output plane with fewer rows than 16-row patches do (heights 12, 24, 36, ...),
// on a tie where the last column of patches can be paired (widths 48, 16, ...: 128->128 at 48^3, N = 2, 0.231 ->
// 0.19 ms), and on a tie where 16-row patches would give a CU fewer than twelve units (more, smaller units balance better).
// Measured, 16 / 12 rows: 256->256 at 24^3 0.119 / 0.100 ms (N = 1), 0.158 / 0.138 (N = 2); 320->320 at 12^3
// 0.083 / 0.070; 128->128 at 48^3 0.152 / 0.130 (N = 1: 4.5 units per CU), 0.243 / 0.231 (N = 2: 9 per CU); 128->64
// at 96^3, N = 2 (27 per CU) 0.666 / 0.691: the large layers lose 1-3 % with 12 rows.
static bool sp_rows12(const Geom& g, int pass) {
    const bool flip = pass == MI3D_PASS_DGRAD;
    const int cout = flip ? g.Cin : g.Cout, Do = flip ? g.D : g.Do, Ho = flip ? g.H : g.Ho, Wo = flip ? g.W : g.Wo;
    const int r16 = (Ho + 15) / 16 * 16, r12 = (Ho + 11) / 12 * 12;
    if (r12 != r16) return r12 < r16;
    // the 12-row build takes a last column of patches that is at most half inside the tensor two patch rows at a time
    const int tail = Wo - (Wo - 1) / 32 * 32;
    if (tail <= 16 && r12 >= 24) return true;
    int dev = 0, cus = 256;
    if (hipGetDevice(&dev) == hipSuccess) (void)hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev);
    const long long units16 = (long long)g.N * (cout / 32) * (r16 / 16) * ((Wo + 31) / 32) * Do;
    return units16 < 12ll * cus;
}

// statistics (mean, 1 / sqrt(var + eps)), or with means = 1 the plain means of the two sums, from partial sums another
// kernel has written in the STATS layout (four waves per workgroup): [workgroup][segment][wave][sum, sum of squares][32 couts], key = sample * CT + cout tile
int sp_stats_finish(const float* part, const int* key, int Cout, int CT, int N, int nwg, int max_seg, double inv_v, float eps, int means,
                    float* stats, hipStream_t s) {
    th16::sp_stats_finish_kernel<<<N * CT, 64 * th16::FIN_SLICES, 0, s>>>(part, key, Cout, CT, nwg, max_seg, inv_v, eps, means, stats);
    return check_launch();
}

bool sp_supported(const Geom& g, int pass) { return th16::supported(g, pass); }
// the chunked variant applies the optional derivative factor of the geometry while it sums the chunks, the other
// variants do in their store path
bool sp_fuses_dgrad_factor(const Geom& g) { return th16::supported(g, MI3D_PASS_DGRAD); }
bool sp_fuses_stats(const Geom& g) { return sp_rows12(g, MI3D_PASS_FWD) ? th12::fuses_stats(g) : th16::fuses_stats(g); }
bool sp_fuses_bwd_sums(const Geom& g) { return sp_rows12(g, MI3D_PASS_DGRAD) ? th12::fuses_bwd_sums(g) : th16::fuses_bwd_sums(g); }
size_t sp_workspace_bytes(const Geom& g, int pass) {
    if (!th16::supported(g, pass)) return 0;
    return sp_rows12(g, pass) ? th12::workspace_bytes(g, pass) : th16::workspace_bytes(g, pass);
}
int sp_conv(const Geom& g, int pass, const void* in, const void* w, void* out, void* ws, size_t ws_bytes, hipStream_t s) {
    return sp_rows12(g, pass) ? th12::conv(g, pass, in, w, out, ws, ws_bytes, s) : th16::conv(g, pass, in, w, out, ws, ws_bytes, s);
}
#endif

}  // namespace mi3d
