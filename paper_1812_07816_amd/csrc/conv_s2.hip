// Forward pass of the 3x3x3 / stride 2 downsampling convolution on bf16 MFMA (v_mfma_f32_32x32x16_bf16), fp32 accumulation: the
// layer that leaves a U-Net level (feature maps of Section 3.1).
//
// The layer moves 64 bytes of input per 27/8 taps, so it is bound by memory
// traffic, not by the matrix cores; the kernel's job is to read every input
// plane once.  Plane streaming as in the stride-1 kernel: a workgroup owns a
// 4-row x 32-col patch of the output plane for up to two 32-wide cout blocks
// and walks along D.  Input plane ip = 2 od - pD + kd feeds output plane od
// through tap kd: planes with even ip + pD feed two output planes (kd 0 and
// 2), odd ones feed one (kd 1); two output planes are in flight in registers.
// The staged plane patch (9 x 65 voxels) is split by column parity in LDS, so
// that the 32 voxels of a fragment (input columns 2 j + kw) are contiguous.
// A kernel instance contracts 32 input channels.  With more input channels the
// 32-channel chunks are separate work units that write fp32 partial outputs, and
// a second kernel adds the chunks in index order and rounds to bf16 (the deep,
// small layers of the encoder: their outputs are a few MB).
#include "mi3d_internal.h"

namespace mi3d {
namespace {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;
typedef __attribute__((__vector_size__(2 * sizeof(float)))) float f32x2;
typedef __attribute__((__vector_size__(2 * sizeof(__bf16)))) __bf16 bf16x2;

constexpr int TH = 4, TW = 32, RH = 2;
constexpr int PC = 2 * TW + 1;                    // staged columns: 65
constexpr int HALF = 33, PITCH = 2 * HALF;        // row pitch in voxels: even columns, then odd columns
constexpr int WB_BYTES = 27 * 2 * 1024;           // packed weights of one 32-wide cout block

struct S2Params {
    const uint16_t* x;
    const uint16_t* wpack;  // [cout block][cin chunk][kw][kd][kh][k16][lane][8]
    uint16_t* y;
    float* part;            // [cin chunk][voxel][Cout] fp32 partial outputs (more than one chunk)
    uint16_t* dump;         // 2 KB that masked store lanes write to instead of y
    int N, D, H, W, Cin, Cout, Do, Ho, Wo, pD, pH, pW;
    int HT, WT, CT, NCH;    // tiles per plane, cout tiles, cin chunks
    long long units;
    int nwg;
    float slope;            // LeakyReLU slope applied to the output (1 = none)
};

__device__ __forceinline__ f32x16 mfma(bf16x8 a, bf16x8 b, f32x16 c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}

// All MFMAs of one staged plane for this wave's two output rows.  The
// accumulator set of output plane m (counted from the segment start) is m % 2.
//   even step (ip + pD even): kd 2 finishes plane m - 1 (set 1 - S), kd 0 starts plane m (set S)
//   odd step: kd 1 continues plane m (set S)
// The six (kw, k16) positions are software-pipelined: the LDS reads of position
// pos + 1 (5 input rows, 6 or 3 weight fragments) are issued before the MFMAs of
// position pos, between scheduling fences; left to itself the compiler emits
// read -> wait -> two MFMAs.  hook(pos) is called once per position: the caller
// spreads its global loads over the step with it.
template <int S, bool EVEN, int SLAB, class Hook>
__device__ __forceinline__ void plane_compute(f32x16 (&acc)[2][RH], const char* in_lane, const char* w_lane, Hook&& hook) {
    constexpr int NKD = EVEN ? 2 : 1;
    bf16x8 xr[2][2 * RH + 1], wf[2][NKD * 3];
    auto load_pos = [&](int pos, int buf) {
        const int kw = pos >> 1, kk = pos & 1;
#pragma unroll
        for (int r = 0; r < 2 * RH + 1; ++r)
            xr[buf][r] = *(const bf16x8*)(in_lane + (2 * kk * SLAB + r * PITCH + (kw & 1) * HALF + (kw >> 1)) * 16);
#pragma unroll
        for (int a = 0; a < NKD; ++a) {
            const int kd = EVEN ? (a == 0 ? 2 : 0) : 1;
#pragma unroll
            for (int kh = 0; kh < 3; ++kh) wf[buf][a * 3 + kh] = *(const bf16x8*)(w_lane + (((kw * 3 + kd) * 3 + kh) * 2 + kk) * 1024);
        }
    };
    load_pos(0, 0);
#pragma unroll
    for (int pos = 0; pos < 6; ++pos) {
        if (pos + 1 < 6) load_pos(pos + 1, (pos + 1) & 1);
#pragma unroll
        for (int kh = 0; kh < 3; ++kh)
#pragma unroll
            for (int a = 0; a < NKD; ++a) {
                const int kd = EVEN ? (a == 0 ? 2 : 0) : 1;
                const int set = (kd == 2) ? 1 - S : S;
#pragma unroll
                for (int r = 0; r < RH; ++r) {
                    if (kd == 0 && pos == 0 && kh == 0) {
                        f32x16 z = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
                        acc[set][r] = mfma(wf[pos & 1][a * 3 + kh], xr[pos & 1][2 * r + kh], z);
                    } else {
                        acc[set][r] = mfma(wf[pos & 1][a * 3 + kh], xr[pos & 1][2 * r + kh], acc[set][r]);
                    }
                }
            }
        hook(pos);
        __builtin_amdgcn_sched_barrier(0);
    }
}

// Stores are unconditional (masked lanes write to the dump area): behind a branch the compiler cannot count
// them and makes the LDS write that follows wait for vmcnt(0), i.e. for the stores themselves.
__device__ __forceinline__ void store_rows(const f32x16 (&a)[RH], uint16_t* p, long long row_pitch, bool col_ok, int rows_ok, uint16_t* dump, float slope) {
    typedef __attribute__((ext_vector_type(2))) unsigned u32x2;
#pragma unroll
    for (int r = 0; r < RH; ++r) {
        uint32_t o[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            f32x2 v = {fmaxf(a[r][2 * i], slope * a[r][2 * i]), fmaxf(a[r][2 * i + 1], slope * a[r][2 * i + 1])};  // LeakyReLU, 0 <= slope <= 1
            bf16x2 b = __builtin_convertvector(v, bf16x2);
            o[i] = __builtin_bit_cast(uint32_t, b);
        }
        uint4 c[2];
#pragma unroll
        for (int k = 0; k < 2; ++k) {
            u32x2 s0 = __builtin_amdgcn_permlane32_swap(o[2 * k], o[2 * k + 4], false, false);
            u32x2 s1 = __builtin_amdgcn_permlane32_swap(o[2 * k + 1], o[2 * k + 5], false, false);
            c[k].x = s0[0]; c[k].y = s1[0]; c[k].z = s0[1]; c[k].w = s1[1];
        }
        uint16_t* q = (col_ok && r < rows_ok) ? p + r * row_pitch : dump;
        *(uint4*)q = c[0];
        *(uint4*)(q + 8) = c[1];
    }
}

// fp32 partial rows: accumulator register i of lane (voxel n, half h) is channel 8 (i / 4) + 4 h + i % 4
__device__ __forceinline__ void store_rows_f32(const f32x16 (&a)[RH], float* p, long long row_pitch, bool col_ok, int rows_ok, float* dump) {
#pragma unroll
    for (int r = 0; r < RH; ++r) {
        float* q = (col_ok && r < rows_ok) ? p + r * row_pitch : dump;
#pragma unroll
        for (int g4 = 0; g4 < 4; ++g4) *(float4*)(q + 8 * g4) = float4{a[r][4 * g4], a[r][4 * g4 + 1], a[r][4 * g4 + 2], a[r][4 * g4 + 3]};
    }
}

// CB = 2 (Cout % 64 == 0): a tile is 4 output rows x 2 cout blocks; waves 0,1 serve block 0 and waves
// 2,3 block 1, two rows each; the staged patch has 9 rows.  CB = 1: 8 output rows x 1 cout block, one
// wave per row pair, 17 staged rows.  The layer is bound by HBM reads and one workgroup per CU holds
// only one plane patch in LDS, so the global loads run two planes ahead of the MFMAs through two
// register sets (plane tq + 2 is requested during step tq and written to LDS at the end of step
// tq + 1): with one plane of lookahead the load latency (about 2 us under load) was exposed in every step.
template <int CB, bool PART>
__global__ void __launch_bounds__(256, 1) s2_fwd_kernel(S2Params P) {
    extern __shared__ __attribute__((aligned(16))) char lds[];
    constexpr int TROWS = CB == 2 ? TH : 2 * TH;      // output rows per workgroup
    constexpr int PR = 2 * TROWS + 1;                 // staged rows
    constexpr int SLAB = PR * PITCH;                  // voxels per 8-channel slab
    constexpr int NPIECE = PR * PC * 4;
    constexpr int NLOAD = (NPIECE + 255) / 256;       // 10 or 18
    constexpr int PER_HOOK = (NLOAD + 5) / 6;
    char* w_lds = lds;
    char* in_lds = lds + CB * WB_BYTES;

    const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
    const int cb = CB == 2 ? (wave >> 1) : 0;
    const int rowgrp = CB == 2 ? (wave & 1) : wave;

    int g = blockIdx.x;
    if ((P.nwg & 7) == 0) g = (g & 7) * (P.nwg >> 3) + (g >> 3);
    long long u0 = P.units * g / P.nwg, u1 = P.units * (g + 1) / P.nwg;

    f32x16 acc[2][RH];
    int lds_off[NLOAD];
#pragma unroll
    for (int i = 0; i < NLOAD; ++i) {
        const int q = t + 256 * i;
        const int v = q >> 2, c = q & 3;
        const int row = (v * 1009) >> 16, col = v - row * PC;  // v / 65 for v < 1200
        lds_off[i] = (c * SLAB + row * PITCH + (col & 1) * HALF + (col >> 1)) * 16;
    }

    int cur_ct = -1;
    while (u0 < u1) {
        long long column = u0 / P.Do;
        const int od_start = (int)(u0 - column * P.Do);
        const long long left = u1 - u0;
        const int od_end = od_start + (int)(left < (long long)(P.Do - od_start) ? left : (long long)(P.Do - od_start));
        u0 += od_end - od_start;
        const int wt = (int)(column % P.WT); column /= P.WT;
        const int ht = (int)(column % P.HT); column /= P.HT;
        const int chunk = PART ? (int)(column % P.NCH) : 0;
        if (PART) column /= P.NCH;
        const int ct = (int)(column % P.CT);
        const int n = (int)(column / P.CT);
        const int h0 = ht * TROWS, w0 = wt * TW;

        __syncthreads();   // previous segment's readers are done with the weights and the stage
        if (ct * P.NCH + chunk != cur_ct) {
            for (int b = 0; b < CB; ++b) {   // the CB cout blocks of the tile, this cin chunk
                const uint4* src = (const uint4*)(P.wpack + ((long long)(ct * CB + b) * P.NCH + chunk) * (WB_BYTES / 2));
                for (int i = t; i < WB_BYTES / 16; i += 256) ((uint4*)(w_lds + b * WB_BYTES))[i] = src[i];
            }
            cur_ct = ct * P.NCH + chunk;
        }
        // load plan: piece q = channels 8c..8c+7 of voxel q / 4 (row-major PR x 65)
        int goff[NLOAD];
        unsigned valid = 0;
#pragma unroll
        for (int i = 0; i < NLOAD; ++i) {
            const int q = t + 256 * i;
            const int v = q >> 2, c = q & 3;
            const int row = (v * 1009) >> 16, col = v - row * PC;
            const int gh = 2 * h0 - P.pH + row, gw = 2 * w0 - P.pW + col;
            const bool ok = q < NPIECE && gh >= 0 && gh < P.H && gw >= 0 && gw < P.W;
            goff[i] = ok ? (gh * P.W + gw) * P.Cin + chunk * 32 + c * 8 : 0;
            valid |= (ok ? 1u : 0u) << i;
        }
        const long long plane_elems = (long long)P.H * P.W * P.Cin;
        const uint16_t* xn = P.x + (long long)n * P.D * plane_elems;
        const long long out_n = (long long)n * P.Do * P.Ho * P.Wo * P.Cout;
        uint16_t* yn = P.y + out_n;
        float* pn = PART ? P.part + (long long)chunk * P.N * P.Do * P.Ho * P.Wo * P.Cout + out_n : nullptr;
        const int nP = od_end - od_start;
        const int nT = 2 * nP + 1;     // staged planes tq = 0 .. 2 nP, input plane ip = 2 od_start - pD + tq
        const int ip0 = 2 * od_start - P.pD;

        // two register sets; loads are unconditional (a plane outside the volume or past the segment
        // reads plane 0 and is zeroed / ignored), so that their waits sit at the LDS writes
        uint4 pre[2][NLOAD];
        unsigned pre_mask[2] = {0u, 0u};
        const uint16_t* pre_base[2] = {xn, xn};
        auto begin_load = [&](int set, int ip) {
            const bool in = ip >= 0 && ip < P.D;
            pre_base[set] = xn + (long long)(in ? ip : 0) * plane_elems;
            pre_mask[set] = in ? valid : 0u;
        };
        auto load_piece = [&](int set, int i) { pre[set][i] = *(const uint4*)(pre_base[set] + goff[i]); };
        auto write_plane = [&](int set) {
#pragma unroll
            for (int i = 0; i < NLOAD; ++i) {
                const bool ok = (pre_mask[set] >> i) & 1;
                uint4 v;
                v.x = ok ? pre[set][i].x : 0u; v.y = ok ? pre[set][i].y : 0u;
                v.z = ok ? pre[set][i].z : 0u; v.w = ok ? pre[set][i].w : 0u;
                if (t + 256 * i < NPIECE) *(uint4*)(in_lds + lds_off[i]) = v;
            }
        };

#pragma unroll
        for (int s = 0; s < 2; ++s)
#pragma unroll
            for (int r = 0; r < RH; ++r)
#pragma unroll
                for (int i = 0; i < 16; ++i) acc[s][r][i] = 0.f;

        begin_load(0, ip0);
#pragma unroll
        for (int i = 0; i < NLOAD; ++i) load_piece(0, i);
        begin_load(1, ip0 + 1);
#pragma unroll
        for (int i = 0; i < NLOAD; ++i) load_piece(1, i);
        write_plane(0);
        __syncthreads();

        const int r0 = rowgrp * RH;            // first output row of this wave within the tile
        const char* in_lane = in_lds + ((lane >> 5) * SLAB + 2 * r0 * PITCH + (lane & 31)) * 16;
        const char* w_lane = w_lds + cb * WB_BYTES + lane * 16;
        const int oh0 = h0 + r0;
        const int ow = w0 + (lane & 31);
        const long long row_pitch = (long long)P.Wo * P.Cout;
        const int co0 = (ct * CB + cb) * 32 + 16 * (lane >> 5);

        // step tq computes staged plane tq (register set tq & 1 is free again: it is refilled with plane
        // tq + 2), then writes plane tq + 1 from the other set.  tq even = 2 m: finishes output plane m - 1.
#define S2_STEP(SET, EVEN)                                                                       \
        {                                                                                        \
            constexpr int rs_ = (EVEN) ? 0 : 1;                                                  \
            begin_load(rs_, ip0 + tq + 2);                                                       \
            plane_compute<SET, EVEN, SLAB>(acc, in_lane, w_lane, [&](int pos) {                  \
                _Pragma("unroll") for (int i_ = 0; i_ < PER_HOOK; ++i_)                          \
                    if (pos * PER_HOOK + i_ < NLOAD) load_piece(rs_, pos * PER_HOOK + i_);       \
            });                                                                                  \
            if (EVEN) {                                                                          \
                const int od_ = od_start + (tq >> 1) - 1;                                        \
                const long long off_ = ((long long)od_ * P.Ho + oh0) * row_pitch + (long long)ow * P.Cout;  \
                if (PART) store_rows_f32(acc[1 - (SET)], pn + off_ + (ct * CB + cb) * 32 + 4 * (lane >> 5), row_pitch, \
                                         tq >= 2 && ow < P.Wo, P.Ho - oh0, (float*)P.dump + lane * 32); \
                else store_rows(acc[1 - (SET)], yn + off_ + co0, row_pitch, tq >= 2 && ow < P.Wo, P.Ho - oh0, P.dump + lane * 16, P.slope); \
            }                                                                                    \
            __syncthreads();                                                                     \
            write_plane(1 - rs_);                                                                \
            __syncthreads();                                                                     \
        }
        for (int tq = 0;;) {
            S2_STEP(0, true)
            if (++tq >= nT) break;
            S2_STEP(0, false)
            if (++tq >= nT) break;
            S2_STEP(1, true)
            if (++tq >= nT) break;
            S2_STEP(1, false)
            if (++tq >= nT) break;
        }
#undef S2_STEP
    }
}

// [Cout][3][3][3][Cin] -> [cout block][cin chunk][kw][kd][kh][k16][lane][8] MFMA A fragments
__global__ void __launch_bounds__(256) s2_pack_weights_kernel(const uint16_t* __restrict__ w, uint16_t* __restrict__ wpack, int Cin, int Cout) {
    long long total = 27ll * Cin * Cout;
    long long idx = (long long)blockIdx.x * 256 + threadIdx.x;
    if (idx >= total) return;
    int j = (int)(idx & 7);
    long long r = idx >> 3;
    int lane = (int)(r & 63); r >>= 6;
    int kk = (int)(r & 1); r >>= 1;
    int kh = (int)(r % 3); r /= 3;
    int kd = (int)(r % 3); r /= 3;
    int kw = (int)(r % 3); r /= 3;
    int nch = Cin / 32;
    int chunk = (int)(r % nch);
    int blk = (int)(r / nch);
    int co = blk * 32 + (lane & 31);
    int ci = chunk * 32 + kk * 16 + 8 * (lane >> 5) + j;
    wpack[idx] = w[((((long long)co * 3 + kd) * 3 + kh) * 3 + kw) * Cin + ci];
}

}  // namespace

// y = bf16(act(sum over chunks of part[chunk])), chunks added in index order; 8 outputs per thread.
// act: LeakyReLU with `slope` (1 = none) if ref is null; otherwise the factor of element i is 1 where
// ref[i] > 0 and `slope` elsewhere (LeakyReLU derivative taken from the activated tensor ref).
__global__ void __launch_bounds__(256) sum_chunks_bf16_kernel(const float* __restrict__ part, uint16_t* __restrict__ y, long long n8, long long n, int nch,
                                                              float slope, const uint16_t* __restrict__ ref, uint16_t* __restrict__ y_hi, int cout,
                                                              const uint16_t* __restrict__ add) {
    typedef __attribute__((__vector_size__(2 * sizeof(float)))) float f32x2_;
    typedef __attribute__((__vector_size__(2 * sizeof(__bf16)))) __bf16 bf16x2_;
    for (long long i = (long long)blockIdx.x * 256 + threadIdx.x; i < n8; i += (long long)gridDim.x * 256) {
        float a[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) a[j] = 0.f;
        for (int c = 0; c < nch; ++c) {
            const float4 lo = *(const float4*)(part + c * n + 8 * i), hi = *(const float4*)(part + c * n + 8 * i + 4);
            a[0] += lo.x; a[1] += lo.y; a[2] += lo.z; a[3] += lo.w; a[4] += hi.x; a[5] += hi.y; a[6] += hi.z; a[7] += hi.w;
        }
        if (add) {   // skip connection: the sum as the plain pass would store it (bf16), plus the second gradient
            const uint4 a4 = *(const uint4*)(add + 8 * i);
            const uint32_t aw[4] = {a4.x, a4.y, a4.z, a4.w};
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                f32x2_ v = {a[2 * j], a[2 * j + 1]};
                const uint32_t r = __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2_));
                a[2 * j] = __builtin_bit_cast(float, r << 16) + __builtin_bit_cast(float, aw[j] << 16);
                a[2 * j + 1] = __builtin_bit_cast(float, r & 0xFFFF0000u) + __builtin_bit_cast(float, aw[j] & 0xFFFF0000u);
            }
        }
        if (ref) {
            const uint4 m4 = *(const uint4*)(ref + 8 * i);
            const uint32_t m[4] = {m4.x, m4.y, m4.z, m4.w};
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                if (!((int)(m[j] << 16) > 0)) a[2 * j] *= slope;
                if (!((int)(m[j] & 0xFFFF0000u) > 0)) a[2 * j + 1] *= slope;
            }
        } else {
#pragma unroll
            for (int j = 0; j < 8; ++j) a[j] = fmaxf(a[j], slope * a[j]);
        }
        uint32_t o[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            f32x2_ v = {a[2 * j], a[2 * j + 1]};
            o[j] = __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2_));
        }
        uint16_t* dst = y + 8 * i;
        if (y_hi) {   // output in two halves of cout / 2 channels per voxel
            const long long vox = 8 * i / cout;
            const int c = (int)(8 * i - vox * cout), half = cout >> 1;
            dst = (c >= half ? y_hi - half : y) + vox * half + c;
        }
        *(uint4*)dst = uint4{o[0], o[1], o[2], o[3]};
    }
}

static size_t s2_part_offset(const Geom& g) { return (((size_t)g.w_elems() * 2 + 255) & ~(size_t)255) + 8192; }

bool s2_fwd_supported(const Geom& g) {
    if (g.dtype != MI3D_BF16 || g.kD != 3 || g.kH != 3 || g.kW != 3) return false;
    if (g.sD != 2 || g.sH != 2 || g.sW != 2) return false;
    if (g.pD > 1 || g.pH > 1 || g.pW > 1) return false;
    if (!g.planes_fit_32bit()) return false;
    return g.Cin % 32 == 0 && g.Cout % 32 == 0;
}

size_t s2_fwd_workspace_bytes(const Geom& g) {
    if (!s2_fwd_supported(g)) return 0;
    size_t b = s2_part_offset(g);   // packed weights + store dump area
    if (g.Cin > 32) b += (size_t)(g.Cin / 32) * g.out_voxels() * g.Cout * sizeof(float);
    return b;
}

int s2_fwd(const Geom& g, const void* x, const void* w, void* y, void* ws, size_t ws_bytes, hipStream_t s) {
    if (ws_bytes < s2_fwd_workspace_bytes(g)) return MI3D_ERR_WORKSPACE;
    long long total = g.w_elems();
    s2_pack_weights_kernel<<<(unsigned)((total + 255) / 256), 256, 0, s>>>((const uint16_t*)w, (uint16_t*)ws, g.Cin, g.Cout);
    int st = check_launch();
    if (st) return st;
    S2Params P;
    P.x = (const uint16_t*)x; P.wpack = (const uint16_t*)ws; P.y = (uint16_t*)y;
    P.dump = (uint16_t*)((char*)ws + (((size_t)g.w_elems() * 2 + 255) & ~(size_t)255));
    P.part = (float*)((char*)ws + s2_part_offset(g));
    P.N = g.N; P.D = g.D; P.H = g.H; P.W = g.W; P.Cin = g.Cin; P.Cout = g.Cout;
    P.Do = g.Do; P.Ho = g.Ho; P.Wo = g.Wo; P.pD = g.pD; P.pH = g.pH; P.pW = g.pW;
    const int CB = (g.Cout % 64 == 0) ? 2 : 1;
    P.CT = g.Cout / (32 * CB);
    P.NCH = g.Cin / 32;
    const int th = CB == 2 ? TH : 2 * TH;
    P.HT = (g.Ho + th - 1) / th;
    P.WT = (g.Wo + TW - 1) / TW;
    P.units = (long long)g.N * P.CT * P.NCH * P.HT * P.WT * g.Do;
    int dev = 0, cus = 256;
    if (hipGetDevice(&dev) == hipSuccess) (void)hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev);
    long long nwg = cus < P.units ? cus : P.units;
    P.nwg = (int)nwg;
    P.slope = g.slope;
    const size_t lds2 = 2 * WB_BYTES + 4 * (2 * TH + 1) * PITCH * 16, lds1 = WB_BYTES + 4 * (4 * TH + 1) * PITCH * 16;
    static std::atomic<bool> attr_set{false};   // set once per process; a second thread racing here repeats an idempotent call
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute((const void*)s2_fwd_kernel<2, false>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds2);
        if (e == hipSuccess) e = hipFuncSetAttribute((const void*)s2_fwd_kernel<1, false>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds1);
        if (e == hipSuccess) e = hipFuncSetAttribute((const void*)s2_fwd_kernel<2, true>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds2);
        if (e == hipSuccess) e = hipFuncSetAttribute((const void*)s2_fwd_kernel<1, true>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds1);
        if (e != hipSuccess) { note_hip_error(e); return MI3D_ERR_HIP; }
        attr_set = true;
    }
    const bool part = P.NCH > 1;
    if (CB == 2 && !part) s2_fwd_kernel<2, false><<<(unsigned)nwg, 256, lds2, s>>>(P);
    else if (CB == 2) s2_fwd_kernel<2, true><<<(unsigned)nwg, 256, lds2, s>>>(P);
    else if (!part) s2_fwd_kernel<1, false><<<(unsigned)nwg, 256, lds1, s>>>(P);
    else s2_fwd_kernel<1, true><<<(unsigned)nwg, 256, lds1, s>>>(P);
    st = check_launch();
    if (st || !part) return st;
    const long long n = (long long)g.out_voxels() * g.Cout;   // Cout % 32 == 0: a multiple of 8
    long long blocks = (n / 8 + 255) / 256;
    if (blocks > 8192) blocks = 8192;
    sum_chunks_bf16_kernel<<<(unsigned)blocks, 256, 0, s>>>(P.part, (uint16_t*)y, n / 8, n, P.NCH, g.slope, nullptr, nullptr, 0, nullptr);
    return check_launch();
}

}  // namespace mi3d
