// Forward pass of the network's first layer: 3x3x3 / stride 1 convolution
// with 4 input channels (the four MRI modalities) on bf16 MFMA.
//
// With Cin = 4 the layer is bound by writing its output (flop/byte 96 against
// a ridge of 312), so the kernel is built around few, wide stores, not around
// MFMA utilisation.  The (kw, ci) pairs of a tap row are folded into the MFMA
// k dimension: k = 4 kw + ci, 12 used of 16, so one v_mfma_f32_32x32x16_bf16
// per (kd, kh) covers 32 voxels x 32 couts.  In NDHWC with 4 channels the 8
// k-values of a lane half are two neighbouring voxels, i.e. 16 contiguous
// bytes of the staged row: fragments need no im2col.  A workgroup computes a
// 16 x 32 patch of one output plane from three input plane patches in LDS;
// two persistent workgroups per CU walk patch columns along D.
#include "mi3d_internal.h"

namespace mi3d {
namespace {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;
typedef __attribute__((__vector_size__(2 * sizeof(float)))) float f32x2;
typedef __attribute__((__vector_size__(2 * sizeof(__bf16)))) __bf16 bf16x2;

constexpr int TH = 16, TW = 32, RH = 4;
constexpr int PR = TH + 2, PCOLS = TW + 3, PITCH = 36;  // patch rows, columns read, row pitch (voxels of 8 bytes)
constexpr int PLANE = PR * PITCH;                        // voxels per staged plane
constexpr int NVOX = PR * PCOLS;                         // voxels to load per plane (630)
constexpr int NLOAD = (NVOX + 255) / 256;                // 3
constexpr int SLOTS = 4;                                 // ring of staged planes: three being read, one being filled

struct C4Params {
    const uint16_t* x;
    const uint16_t* wpack;  // [cout block][kd][kh][lane][8]
    uint16_t* y;
    uint16_t* dump;         // 4 KB that masked store lanes write to instead of y
    int N, D, H, W, Cout, Do, Ho, Wo, pD, pH, pW, HT, WT;
    long long tiles;        // N*HT*WT*Do, output plane fastest
    int nwg;
    float slope;            // LeakyReLU slope applied to the output (1 = none)
    // STATS: per-(workgroup, segment, wave) sums of y and y^2 over the voxels, 32 couts each, in the layout of the
    // plane-streaming kernel's statistics: [workgroup][segment][wave][sum, sum of squares][32]; key = sample, -1 = unused
    float* stat_part;
    int* stat_key;
    int max_seg;
};

// Persistent workgroups walk a contiguous range of (n, 16-row, 32-col, od) tiles, output plane fastest: a
// workgroup moves along D through one patch column and keeps the input planes in a ring of four LDS slots, so
// that every input plane of a segment is fetched once (three planes at the start of a segment, then one per
// tile, loaded into registers while the current tile is computed and stored).
// ONE: Cout == 32, the 9 weight fragments stay in registers for the whole kernel (otherwise they are
// re-read from L2 for every cout block of every tile, a load latency per tile that nothing hides)
// STATS (with ONE): the kernel also adds up y and y^2 per output channel (of the bf16 values it stores) for the instance
// normalisation that follows the layer (Section 4.1): a lane stores the same 8 couts of every voxel it handles, keeps
// their sums over a segment, and the 16 lanes that share the couts add theirs in a fixed butterfly.
template <bool ONE, bool STATS = false>
__global__ void __launch_bounds__(256, 2) c4_fwd_kernel(C4Params P) {
    // ring of planes, 1 KB that threads without a voxel of the plane write to, store staging
    __shared__ __attribute__((aligned(16))) char lds[SLOTS * PLANE * 8 + 1024 + 4 * RH * 2048];
    const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
    bf16x8 wf[9];
    if (ONE) {
#pragma unroll
        for (int q = 0; q < 9; ++q) wf[q] = ((const bf16x8*)P.wpack)[q * 64 + lane];
    }
    char* stg = lds + SLOTS * PLANE * 8 + 1024 + wave * RH * 2048;  // this wave's store staging: RH rows x 32 voxels x 64 B
    // Work split.  With at least as many workgroups as patch columns, workgroup g takes column g % columns and
    // the g / columns-th of S equal D segments: workgroups that run side by side then write neighbouring patches of
    // the same few planes, and every workgroup streams along D for its whole range so the ring of staged planes is
    // primed once.  Otherwise contiguous ranges of tiles.
    long long u, u1;
    const long long columns = P.tiles / P.Do;
    if (P.nwg >= columns) {
        const int S = (int)(P.nwg / columns);
        const int seg = (int)(blockIdx.x / columns);
        const long long col = blockIdx.x % columns;
        if (seg >= S) {
            if (STATS && t == 0)
                for (int k = 0; k < P.max_seg; ++k) P.stat_key[blockIdx.x * P.max_seg + k] = -1;
            return;
        }
        u = col * P.Do + (long long)P.Do * seg / S;
        u1 = col * P.Do + (long long)P.Do * (seg + 1) / S;
    } else {
        u = P.tiles * blockIdx.x / P.nwg;
        u1 = P.tiles * (blockIdx.x + 1) / P.nwg;
    }

    // this thread's voxels of a staged plane: row, column and LDS offset are the same for every plane
    int prow[NLOAD], pcol[NLOAD], lds_off[NLOAD];
#pragma unroll
    for (int i = 0; i < NLOAD; ++i) {
        const int q = t + 256 * i;
        prow[i] = q / PCOLS;
        pcol[i] = q - prow[i] * PCOLS;
        lds_off[i] = q < NVOX ? (prow[i] * PITCH + pcol[i]) * 8 : -1;
    }

    int seg_i = 0;   // STATS: index of the segment within this workgroup's range
    while (u < u1) {
        long long b = u / P.Do;
        const int od0 = (int)(u - b * P.Do);
        const long long left = u1 - u;
        const int od1 = left < (long long)(P.Do - od0) ? od0 + (int)left : P.Do;
        u += od1 - od0;
        const int wt = (int)(b % P.WT); b /= P.WT;
        const int ht = (int)(b % P.HT);
        const int n = (int)(b / P.HT);
        const int h0 = ht * TH, w0 = wt * TW;

        // plane q of the ring is input plane gd = q - pD (zero outside the volume), kept in slot q % 4
        long long voff[NLOAD];
        bool vok[NLOAD];
#pragma unroll
        for (int i = 0; i < NLOAD; ++i) {
            const int gh = h0 - P.pH + prow[i], gw = w0 - P.pW + pcol[i];
            vok[i] = t + 256 * i < NVOX && gh >= 0 && gh < P.H && gw >= 0 && gw < P.W;
            voff[i] = vok[i] ? ((long long)gh * P.W + gw) * 4 : 0;
        }
        const uint16_t* xn = P.x + (long long)n * P.D * P.H * P.W * 4;
        const long long plane_elems = (long long)P.H * P.W * 4;
        // Loads and LDS writes are unconditional: voxels outside the volume read a valid address and are zeroed when
        // they are written, threads without a voxel write to the spare KB.  Behind a branch the compiler cannot pair
        // a load with its use and waits for vmcnt(0), i.e. for the stores of the tile as well.
        uint2 px[NLOAD];
        bool pin = false;
        auto load_plane = [&](int q) {
            const int gd = q - P.pD;
            pin = gd >= 0 && gd < P.D;
            const uint16_t* base = xn + (pin ? gd : 0) * plane_elems;
#pragma unroll
            for (int i = 0; i < NLOAD; ++i) px[i] = *(const uint2*)(base + voff[i]);
        };
        auto write_plane = [&](int q) {
            char* dst = lds + (q & (SLOTS - 1)) * PLANE * 8;
#pragma unroll
            for (int i = 0; i < NLOAD; ++i) {
                const bool keep = pin && vok[i];
                const uint2 v = {keep ? px[i].x : 0u, keep ? px[i].y : 0u};
                char* w = lds_off[i] >= 0 ? dst + lds_off[i] : lds + SLOTS * PLANE * 8 + (t & 127) * 8;
                *(uint2*)w = v;
            }
        };

        __syncthreads();  // readers of the previous segment are done
        for (int kd = 0; kd < 3; ++kd) {
            load_plane(od0 + kd);
            write_plane(od0 + kd);
        }
        __syncthreads();

        // Registers that hold the data of the tile's global stores.  The compiler makes whoever writes a register
        // next wait until the store that read it has completed; left to the allocator these registers are reused
        // right at the top of the next tile, which then waits a full store latency.  The empty asm below keeps them
        // allocated until the next tile's own data replaces them, when those stores are long done.
        typedef __attribute__((ext_vector_type(4))) unsigned u32x4;
        u32x4 ov[2 * RH];
#pragma unroll
        for (int i = 0; i < 2 * RH; ++i) ov[i] = u32x4{0u, 0u, 0u, 0u};
        float st1[STATS ? 8 : 1], st2[STATS ? 8 : 1];
        if constexpr (STATS) {
#pragma unroll
            for (int j = 0; j < 8; ++j) st1[j] = st2[j] = 0.f;
        }
        for (int od = od0; od < od1; ++od) {
            load_plane(od + 3);  // the plane the next tile adds (after the last tile: fetched, never read)
            __builtin_amdgcn_sched_barrier(0);  // keeps the loads here, a whole tile ahead of the LDS write that uses them

            // input fragments: lane (voxel n, half h) holds voxels n + 2h and n + 2h + 1 of the row = taps kw 2h, 2h + 1
            bf16x8 xf[3][RH + 2];
            const char* xl = lds + (wave * RH * PITCH + (lane & 31) + 2 * (lane >> 5)) * 8;
#pragma unroll
            for (int kd = 0; kd < 3; ++kd) {
                const char* xs = xl + ((od + kd) & (SLOTS - 1)) * PLANE * 8;
#pragma unroll
                for (int r = 0; r < RH + 2; ++r) {
                    const uint2 lo = *(const uint2*)(xs + (r * PITCH) * 8);
                    const uint2 hi = *(const uint2*)(xs + (r * PITCH + 1) * 8);
                    const uint4 v = {lo.x, lo.y, hi.x, hi.y};
                    xf[kd][r] = __builtin_bit_cast(bf16x8, v);
                }
            }

            const int oh0 = h0 + wave * RH;
            const long long row_pitch = (long long)P.Wo * P.Cout;
            uint16_t* ybase = P.y + ((((long long)n * P.Do + od) * P.Ho + oh0) * P.Wo + w0) * P.Cout;

            for (int cb = 0; cb < (ONE ? 1 : P.Cout / 32); ++cb) {
                if (!ONE) {
                    const bf16x8* wp = (const bf16x8*)(P.wpack + (long long)cb * 9 * 512) + lane;
#pragma unroll
                    for (int q = 0; q < 9; ++q) wf[q] = wp[q * 64];
                }
                f32x16 acc[RH];
#pragma unroll
                for (int kd = 0; kd < 3; ++kd)
#pragma unroll
                    for (int kh = 0; kh < 3; ++kh)
#pragma unroll
                        for (int r = 0; r < RH; ++r) {
                            if (kd == 0 && kh == 0) {
                                f32x16 z = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
                                acc[r] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf[0], xf[0][r], z, 0, 0, 0);
                            } else {
                                acc[r] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf[kd * 3 + kh], xf[kd][r + kh], acc[r], 0, 0, 0);
                            }
                        }
                typedef __attribute__((ext_vector_type(2))) unsigned u32x2;
                // lane (n, h) ends with couts 16h .. 16h+15 of voxel n; the rows pass through LDS so that
                // each store instruction writes whole 64-byte voxels of 16 neighbouring voxels
                __builtin_amdgcn_wave_barrier();
#pragma unroll
                for (int r = 0; r < RH; ++r) {
                    uint32_t o[8];
#pragma unroll
                    for (int i = 0; i < 8; ++i) {
                        f32x2 v = {fmaxf(acc[r][2 * i], P.slope * acc[r][2 * i]), fmaxf(acc[r][2 * i + 1], P.slope * acc[r][2 * i + 1])};  // LeakyReLU, 0 <= slope <= 1
                        bf16x2 bb = __builtin_convertvector(v, bf16x2);
                        o[i] = __builtin_bit_cast(uint32_t, bb);
                    }
                    uint4 c[2];
#pragma unroll
                    for (int k = 0; k < 2; ++k) {
                        u32x2 s0 = __builtin_amdgcn_permlane32_swap(o[2 * k], o[2 * k + 4], false, false);
                        u32x2 s1 = __builtin_amdgcn_permlane32_swap(o[2 * k + 1], o[2 * k + 5], false, false);
                        c[k].x = s0[0]; c[k].y = s1[0]; c[k].z = s0[1]; c[k].w = s1[1];
                    }
                    char* q = stg + r * 2048 + (lane & 31) * 64 + (lane >> 5) * 32;
                    *(uint4*)q = c[0];
                    *(uint4*)(q + 16) = c[1];
                }
                // same wave, LDS executes in order: only the compiler must not move the reads above the writes
                asm volatile("" ::: "memory");
                __builtin_amdgcn_wave_barrier();
                asm volatile("" ::: "memory");
#pragma unroll
                for (int i = 0; i < 2 * RH; ++i) asm volatile("" ::"v"(ov[i]));
#pragma unroll
                for (int r = 0; r < RH; ++r)
#pragma unroll
                    for (int i = 0; i < 2; ++i) {
                        const u32x4 v = ov[2 * r + i] = *(const u32x4*)(stg + r * 2048 + i * 1024 + lane * 16);
                        const int vox = i * 16 + (lane >> 2);
                        // unconditional (masked lanes write to the dump area): the compiler can then count the stores and
                        // lets them fly while the next plane goes to LDS, instead of waiting for vmcnt(0) every tile
                        const bool inside = w0 + vox < P.Wo && oh0 + r < P.Ho;
                        uint16_t* dst = inside ? ybase + r * row_pitch + (long long)vox * P.Cout + cb * 32 + (lane & 3) * 8 : P.dump + t * 8;
                        *(u32x4*)dst = v;
                        if constexpr (STATS) {
                            const unsigned wv[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
                            for (int j = 0; j < 4; ++j) {
                                const unsigned q = inside ? wv[j] : 0u;
                                const float lo = __builtin_bit_cast(float, q << 16), hi = __builtin_bit_cast(float, q & 0xffff0000u);
                                st1[2 * j] += lo; st2[2 * j] = fmaf(lo, lo, st2[2 * j]);
                                st1[2 * j + 1] += hi; st2[2 * j + 1] = fmaf(hi, hi, st2[2 * j + 1]);
                            }
                        }
                    }
            }
            // the slot of plane od + 3 held plane od - 1, whose readers passed the barrier of the previous tile
            __builtin_amdgcn_sched_barrier(0);  // the use of the loaded plane stays down here, behind the tile's work
            write_plane(od + 3);
            __syncthreads();
        }
        if constexpr (STATS) {
            // lanes l, l + 4, l + 8, ... hold the same couts 8 (l % 4) .. 8 (l % 4) + 7
#pragma unroll
            for (int j = 0; j < 8; ++j)
#pragma unroll
                for (int off = 32; off >= 4; off >>= 1) {
                    st1[j] += __shfl_xor(st1[j], off, 64);
                    st2[j] += __shfl_xor(st2[j], off, 64);
                }
            if (t == 0) P.stat_key[blockIdx.x * P.max_seg + seg_i] = n;
            if (lane < 4) {
                float* out = P.stat_part + (((long long)blockIdx.x * P.max_seg + seg_i) * 4 + wave) * 64;
#pragma unroll
                for (int j = 0; j < 8; ++j) {
                    out[8 * lane + j] = st1[j];
                    out[32 + 8 * lane + j] = st2[j];
                }
            }
            ++seg_i;
        }
    }
    if constexpr (STATS) {
        if (t == 0)
            for (; seg_i < P.max_seg; ++seg_i) P.stat_key[blockIdx.x * P.max_seg + seg_i] = -1;   // unused slots of this workgroup
    }
}

// [Cout][3][3][3][4] -> [cout block][kd][kh][lane][8]: lane (co, half h) holds k = 8h + j = (kw = 2h + j/4, ci = j%4)
__global__ void __launch_bounds__(256) c4_pack_weights_kernel(const uint16_t* __restrict__ w, uint16_t* __restrict__ wpack, int Cout) {
    const long long total = (long long)(Cout / 32) * 9 * 512;
    const long long idx = (long long)blockIdx.x * 256 + threadIdx.x;
    if (idx >= total) return;
    const int j = (int)(idx & 7);
    long long r = idx >> 3;
    const int lane = (int)(r & 63); r >>= 6;
    const int kh = (int)(r % 3); r /= 3;
    const int kd = (int)(r % 3); r /= 3;
    const int cb = (int)r;
    const int co = cb * 32 + (lane & 31);
    const int kw = 2 * (lane >> 5) + (j >> 2), ci = j & 3;
    wpack[idx] = kw < 3 ? w[((((long long)co * 3 + kd) * 3 + kh) * 3 + kw) * 4 + ci] : (uint16_t)0;
}

}  // namespace

bool c4_fwd_supported(const Geom& g) {
    if (g.dtype != MI3D_BF16 || g.kD != 3 || g.kH != 3 || g.kW != 3) return false;
    if (g.sD != 1 || g.sH != 1 || g.sW != 1) return false;
    if (g.pD > 2 || g.pH > 2 || g.pW > 2) return false;
    if (!g.planes_fit_32bit()) return false;
    return g.Cin == 4 && g.Cout % 32 == 0;
}

// workgroups and the most segments (runs along D inside one patch column) one of them walks
static void c4_fwd_layout(const Geom& g, long long* tiles, int* nwg, int* max_seg) {
    *tiles = (long long)g.N * ((g.Ho + TH - 1) / TH) * ((g.Wo + TW - 1) / TW) * g.Do;
    *nwg = (int)(*tiles < 512 ? *tiles : 512);
    const long long columns = *tiles / g.Do;
    if (*nwg >= columns) *max_seg = 1;
    else *max_seg = (int)(((*tiles + *nwg - 1) / *nwg + g.Do - 1) / g.Do) + 1;
}

bool c4_fwd_fuses_stats(const Geom& g) { return c4_fwd_supported(g) && g.Cout == 32; }

size_t c4_fwd_workspace_bytes(const Geom& g) {
    if (!c4_fwd_supported(g)) return 0;
    long long tiles; int nwg, max_seg;
    c4_fwd_layout(g, &tiles, &nwg, &max_seg);
    // packed weights, store dump area, partial sums and keys of the variant with statistics
    return (size_t)(g.Cout / 32) * 9 * 1024 + 4096 + (size_t)nwg * max_seg * (4 * 64 * sizeof(float) + sizeof(int)) + 256;
}

int c4_fwd(const Geom& g, const void* x, const void* w, void* y, void* ws, size_t ws_bytes, hipStream_t s) {
    if (ws_bytes < c4_fwd_workspace_bytes(g)) return MI3D_ERR_WORKSPACE;
    const long long total = (long long)(g.Cout / 32) * 9 * 512;
    c4_pack_weights_kernel<<<(unsigned)((total + 255) / 256), 256, 0, s>>>((const uint16_t*)w, (uint16_t*)ws, g.Cout);
    int st = check_launch();
    if (st) return st;
    C4Params P;
    P.x = (const uint16_t*)x; P.wpack = (const uint16_t*)ws; P.y = (uint16_t*)y;
    P.dump = (uint16_t*)((char*)ws + (size_t)(g.Cout / 32) * 9 * 1024);
    P.N = g.N; P.D = g.D; P.H = g.H; P.W = g.W; P.Cout = g.Cout;
    P.Do = g.Do; P.Ho = g.Ho; P.Wo = g.Wo; P.pD = g.pD; P.pH = g.pH; P.pW = g.pW;
    P.HT = (g.Ho + TH - 1) / TH;
    P.WT = (g.Wo + TW - 1) / TW;
    c4_fwd_layout(g, &P.tiles, &P.nwg, &P.max_seg);
    P.slope = g.slope;
    P.stat_part = (float*)((char*)ws + (size_t)(g.Cout / 32) * 9 * 1024 + 4096);
    P.stat_key = (int*)(P.stat_part + (size_t)P.nwg * P.max_seg * 4 * 64);
    if (g.stats) {
        if (!c4_fwd_fuses_stats(g)) return MI3D_ERR_UNSUPPORTED;
        c4_fwd_kernel<true, true><<<(unsigned)P.nwg, 256, 0, s>>>(P);
        st = check_launch();
        if (st) return st;
        return sp_stats_finish(P.stat_part, P.stat_key, 32, 1, g.N, P.nwg, P.max_seg, 1.0 / ((double)g.Do * g.Ho * g.Wo), g.stats_eps, 0, g.stats, s);
    }
    if (g.Cout == 32) c4_fwd_kernel<true><<<(unsigned)P.nwg, 256, 0, s>>>(P);
    else c4_fwd_kernel<false><<<(unsigned)P.nwg, 256, 0, s>>>(P);
    return check_launch();
}

}  // namespace mi3d

// ---------------------------------------------------------------------------
// Weight gradient of the same layer: dw[co,t,ci] = sum_v dy[v,co] * x[v + t - p, ci].
// The contraction runs over voxels; (kw, ci) is folded into the MFMA n
// dimension (12 of 16 used), so one v_mfma_f32_16x16x32_bf16 per (kd, kh)
// covers 16 couts x 32 voxels.  Both operands come from transposing LDS reads;
// for x each lane passes the address of the voxel shifted by its own kw, so
// the staged rows need no rearrangement.  A workgroup walks a contiguous range
// of 16 x 32 dy patches, plane after plane along D for one patch position, and
// keeps the three x planes of a patch as a ring in LDS: from one patch to the
// next along D only one new x plane is fetched.  It keeps its 9 accumulators
// per wave in registers and writes one partial-sum slot per wave pair; a second
// kernel adds the slots in index order (bit-reproducible) and drops the padding
// columns.
namespace mi3d {
namespace {

typedef __attribute__((__vector_size__(4 * sizeof(short)))) short s16x4;
typedef __attribute__((__vector_size__(8 * sizeof(short)))) short s16x8;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float f32x4;

constexpr int WDY_SLAB = TH * TW * 32;          // one 16-cout slab of the dy patch
constexpr int WDY_BYTES = 2 * WDY_SLAB;         // 32 KB
constexpr int NVOX3 = 3 * PR * PCOLS;           // voxels of a three-plane x patch (1890)
constexpr int NLOAD3 = (NVOX3 + 255) / 256;      // 8
constexpr int WX_BYTES = 3 * PLANE * 8;         // 15.2 KB
constexpr int WNDY = TH * TW * 4 / 256;         // 8 16-byte pieces per thread

struct C4WgParams {
    const uint16_t* x;
    const uint16_t* dy;
    float* part;   // [slot][Cout][9][16]
    int N, D, H, W, Cout, Do, Ho, Wo, pD, pH, pW, HT, WT;
    long long tiles;  // N*HT*WT*Do, the plane index running fastest
    int nwg;
};

__device__ __forceinline__ int c4_mod3(int v) { return ((v % 3) + 3) % 3; }

__device__ __forceinline__ bf16x8 tr8(const char* p0, const char* p1) {
    typedef __attribute__((address_space(3))) s16x4* lptr;
    s16x4 a = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lptr)p0);
    s16x4 b = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lptr)p1);
    s16x8 c = __builtin_shufflevector(a, b, 0, 1, 2, 3, 4, 5, 6, 7);
    return __builtin_bit_cast(bf16x8, c);
}

__global__ void __launch_bounds__(256, 2) c4_wgrad_kernel(C4WgParams P) {
    __shared__ __attribute__((aligned(16))) char lds[WX_BYTES + WDY_BYTES];
    char* x_lds = lds;
    char* dy_lds = lds + WX_BYTES;
    const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
    const int coh = wave & 1, rh = wave >> 1;   // 16-cout half, half of the patch rows
    const int cot = blockIdx.y;
    const long long t0 = P.tiles * blockIdx.x / P.nwg, t1 = P.tiles * (blockIdx.x + 1) / P.nwg;

    const int g = lane >> 4, s = lane & 15;
    // dy: lane supplies voxel 4g + s/4 (+16), couts 4(s%4)..+3 of the wave's 16-cout slab
    const char* dy_lane = dy_lds + coh * WDY_SLAB + (4 * g + (s >> 2)) * 32 + (s & 3) * 8;
    // x: lane supplies voxel 4g + s/4 (+16) shifted by kw = s%4, all 4 channels
    const char* x_lane = x_lds + (4 * g + (s >> 2) + (s & 3)) * 8;

    f32x4 acc[3][3];
#pragma unroll
    for (int a = 0; a < 3; ++a)
#pragma unroll
        for (int b = 0; b < 3; ++b) acc[a][b] = f32x4{0.f, 0.f, 0.f, 0.f};

    // patch loads of one tile into registers (zero outside the volume)
    uint2 px[NLOAD3];
    uint4 pdy[WNDY];
    // A tile that continues the previous one along D (same patch position, next plane) needs only the x plane of
    // tap kd = 2; the other two are in the ring already.
    auto continues = [&](long long tile) { return tile > t0 && tile % P.Do != 0; };
    auto load_tile = [&](long long tile) {
        long long b = tile;
        const int od = (int)(b % P.Do); b /= P.Do;
        const int wt = (int)(b % P.WT); b /= P.WT;
        const int ht = (int)(b % P.HT);
        const int n = (int)(b / P.HT);
        const int h0 = ht * TH, w0 = wt * TW;
        const int first_pl = continues(tile) ? 2 : 0;
#pragma unroll
        for (int i = 0; i < NLOAD3; ++i) {
            const int q = t + 256 * i;
            const int pl = q / (PR * PCOLS), rem = q - pl * (PR * PCOLS);
            const int row = rem / PCOLS, col = rem - row * PCOLS;
            const int gd = od - P.pD + pl, gh = h0 - P.pH + row, gw = w0 - P.pW + col;
            px[i] = uint2{0u, 0u};
            if (q < NVOX3 && pl >= first_pl && gd >= 0 && gd < P.D && gh >= 0 && gh < P.H && gw >= 0 && gw < P.W)
                px[i] = *(const uint2*)(P.x + ((((long long)n * P.D + gd) * P.H + gh) * P.W + gw) * 4);
        }
#pragma unroll
        for (int i = 0; i < WNDY; ++i) {
            const int q = t + 256 * i, v = q >> 2, c = q & 3;
            const int gh = h0 + (v >> 5), gw = w0 + (v & 31);
            pdy[i] = uint4{0u, 0u, 0u, 0u};
            if (gh < P.Ho && gw < P.Wo)
                pdy[i] = *(const uint4*)(P.dy + ((((long long)n * P.Do + od) * P.Ho + gh) * P.Wo + gw) * P.Cout + cot * 32 + c * 8);
        }
    };
    // x plane ip of a patch lives in ring slot ip mod 3
    auto write_tile = [&](long long tile) {
        const int ip0 = (int)(tile % P.Do) - P.pD;
        const int first_pl = continues(tile) ? 2 : 0;
#pragma unroll
        for (int i = 0; i < NLOAD3; ++i) {
            const int q = t + 256 * i;
            const int pl = q / (PR * PCOLS), rem = q - pl * (PR * PCOLS);
            const int row = rem / PCOLS, col = rem - row * PCOLS;
            if (q < NVOX3 && pl >= first_pl) *(uint2*)(x_lds + (c4_mod3(ip0 + pl) * PLANE + row * PITCH + col) * 8) = px[i];
        }
#pragma unroll
        for (int i = 0; i < WNDY; ++i) {
            const int q = t + 256 * i, v = q >> 2, c = q & 3;
            *(uint4*)(dy_lds + (c >> 1) * WDY_SLAB + v * 32 + (c & 1) * 16) = pdy[i];
        }
    };

    if (t0 < t1) load_tile(t0);
    for (long long tile = t0; tile < t1; ++tile) {
        __syncthreads();  // readers of the previous tile are done
        write_tile(tile);
        __syncthreads();
        if (tile + 1 < t1) load_tile(tile + 1);  // in flight during the MFMA work below

        // this wave's 8 dy rows, then every x row that meets them
        const int ip0 = (int)(tile % P.Do) - P.pD;
        bf16x8 dyf[TH / 2];
#pragma unroll
        for (int r = 0; r < TH / 2; ++r) {
            const char* p = dy_lane + (rh * (TH / 2) + r) * TW * 32;
            dyf[r] = tr8(p, p + 16 * 32);
        }
#pragma unroll
        for (int kd = 0; kd < 3; ++kd)
#pragma unroll
            for (int rr = 0; rr < TH / 2 + 2; ++rr) {
                const char* p = x_lane + (c4_mod3(ip0 + kd) * PLANE + (rh * (TH / 2) + rr) * PITCH) * 8;
                const bf16x8 xf = tr8(p, p + 16 * 8);
#pragma unroll
                for (int kh = 0; kh < 3; ++kh) {
                    const int dr = rr - kh;
                    if (dr < 0 || dr >= TH / 2) continue;
                    acc[kd][kh] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(dyf[dr], xf, acc[kd][kh], 0, 0, 0);
                }
            }
    }

    // add the two row halves (fixed order: upper half onto lower), then one slot per workgroup.
    // acc register v of lane l: co = 4 (l / 16) + v of the wave's half, n = l % 16 = 4 kw + ci
    __syncthreads();
    float* red = (float*)lds;  // [coh][kd*3+kh][v][lane]
    if (rh == 1) {
#pragma unroll
        for (int q = 0; q < 9; ++q)
#pragma unroll
            for (int v = 0; v < 4; ++v) red[((coh * 9 + q) * 4 + v) * 64 + lane] = acc[q / 3][q % 3][v];
    }
    __syncthreads();
    if (rh == 0) {
        float* out = P.part + ((long long)blockIdx.x * P.Cout + cot * 32 + coh * 16) * 144;
#pragma unroll
        for (int q = 0; q < 9; ++q)
#pragma unroll
            for (int v = 0; v < 4; ++v)
                out[((4 * (lane >> 4) + v) * 9 + q) * 16 + (lane & 15)] = acc[q / 3][q % 3][v] + red[((coh * 9 + q) * 4 + v) * 64 + lane];
    }
}

// dw[co][kd][kh][kw][0..3] = sum over slots of part[slot][co][kd*3+kh][4 kw + 0..3]; a block handles four
// (co, kd, kh, kw) positions, thread (g, e) adds the four channels of slots g, g + 64, ... of position e; the 64 group
// sums are then added in index order (a fixed order: bit-reproducible)
__global__ void __launch_bounds__(256) c4_wgrad_reduce_kernel(const float* __restrict__ part, float* __restrict__ dw, int Cout, int slots) {
    __shared__ float4 sm[64][4];
    const int e = threadIdx.x & 3, g = threadIdx.x >> 2;
    const int idx = blockIdx.x * 4 + e;            // (co, kdh, kw)
    const bool ok = idx < Cout * 27;
    int r = idx;
    const int kw = r % 3; r /= 3;
    const int kdh = r % 9;
    const int co = r / 9;
    float4 a = make_float4(0.f, 0.f, 0.f, 0.f);
    if (ok)
        for (int sl = g; sl < slots; sl += 64) {
            const float4 b = *(const float4*)(part + (((long long)sl * Cout + co) * 9 + kdh) * 16 + 4 * kw);
            a.x += b.x; a.y += b.y; a.z += b.z; a.w += b.w;
        }
    sm[g][e] = a;
    __syncthreads();
    if (g == 0 && ok) {
        float4 b = make_float4(0.f, 0.f, 0.f, 0.f);
        for (int k = 0; k < 64; ++k) {
            const float4 c = sm[k][e];
            b.x += c.x; b.y += c.y; b.z += c.z; b.w += c.w;
        }
        *(float4*)(dw + 4 * (long long)idx) = b;
    }
}

}  // namespace

bool c4_wgrad_supported(const Geom& g) { return c4_fwd_supported(g); }

static int c4_wgrad_nwg(const Geom& g) {
    const long long tiles = (long long)g.N * g.Do * ((g.Ho + TH - 1) / TH) * ((g.Wo + TW - 1) / TW);
    const long long cap = 512 / (g.Cout / 32) > 0 ? 512 / (g.Cout / 32) : 1;
    return (int)(tiles < cap ? tiles : cap);
}

size_t c4_wgrad_workspace_bytes(const Geom& g) {
    if (!c4_wgrad_supported(g)) return 0;
    return (size_t)c4_wgrad_nwg(g) * g.Cout * 144 * sizeof(float);
}

int c4_wgrad(const Geom& g, const void* x, const void* dy, float* dw, void* ws, size_t ws_bytes, hipStream_t s) {
    if (ws_bytes < c4_wgrad_workspace_bytes(g)) return MI3D_ERR_WORKSPACE;
    C4WgParams P;
    P.x = (const uint16_t*)x; P.dy = (const uint16_t*)dy; P.part = (float*)ws;
    P.N = g.N; P.D = g.D; P.H = g.H; P.W = g.W; P.Cout = g.Cout;
    P.Do = g.Do; P.Ho = g.Ho; P.Wo = g.Wo; P.pD = g.pD; P.pH = g.pH; P.pW = g.pW;
    P.HT = (g.Ho + TH - 1) / TH;
    P.WT = (g.Wo + TW - 1) / TW;
    P.tiles = (long long)g.N * P.HT * P.WT * g.Do;
    P.nwg = c4_wgrad_nwg(g);
    c4_wgrad_kernel<<<dim3((unsigned)P.nwg, (unsigned)(g.Cout / 32)), 256, 0, s>>>(P);
    int st = check_launch();
    if (st) return st;
    c4_wgrad_reduce_kernel<<<(unsigned)((g.Cout * 27 + 3) / 4), 256, 0, s>>>((const float*)ws, dw, g.Cout, P.nwg);
    return check_launch();
}

}  // namespace mi3d
