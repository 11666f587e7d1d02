// Diagnostic: the rate of a bare v_mfma_f32_32x32x16_bf16 (and v_mfma_f32_32x32x2_f32) loop on this device, with operands
// held in registers.
// The MFMA-bound convolution kernels are limited by power, and the power of an MFMA depends on its operands: with
// all-zero operands the loop reaches the published dense peak, with random operands about 70 % of it.  bench.py
// reports both next to the convolution kernels' rates, so that their distance from what the matrix cores sustain
// on real data can be told from their distance from the published peak.
// Measurement-side helper: built into libbench_probe.so next to bench.py, not part of libmi3d.so or its C ABI.
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

namespace {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;

// 4 waves per workgroup, one workgroup per CU; each wave keeps 12 independent accumulators (as the plane-streaming
// convolution does) and four A and four B fragments loaded once from `in` (4096 16-byte pieces).
__global__ void __launch_bounds__(256, 1) mfma_rate_kernel(const uint4* __restrict__ in, float* __restrict__ out, int iters) {
    bf16x8 a[4], b[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        a[i] = __builtin_bit_cast(bf16x8, in[(threadIdx.x * 8 + i) & 4095]);
        b[i] = __builtin_bit_cast(bf16x8, in[(threadIdx.x * 8 + 4 + i) & 4095]);
    }
    f32x16 acc[12];
#pragma unroll
    for (int k = 0; k < 12; ++k)
#pragma unroll
        for (int j = 0; j < 16; ++j) acc[k][j] = 0.f;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int k = 0; k < 12; ++k) acc[k] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[k & 3], b[(k + 1) & 3], acc[k], 0, 0, 0);
    }
    float s = 0.f;
#pragma unroll
    for (int k = 0; k < 12; ++k)
#pragma unroll
        for (int j = 0; j < 16; ++j) s += acc[k][j];
    out[blockIdx.x * 256 + threadIdx.x] = s;
}

// The same loop for the fp32 matrix cores (v_mfma_f32_32x32x2_f32: one float of each operand per lane)
__global__ void __launch_bounds__(256, 1) mfma_rate_f32_kernel(const float* __restrict__ in, float* __restrict__ out, int iters) {
    float a[4], b[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        a[i] = in[(threadIdx.x * 8 + i) & 16383];
        b[i] = in[(threadIdx.x * 8 + 4 + i) & 16383];
    }
    f32x16 acc[12];
#pragma unroll
    for (int k = 0; k < 12; ++k)
#pragma unroll
        for (int j = 0; j < 16; ++j) acc[k][j] = 0.f;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int k = 0; k < 12; ++k) acc[k] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[k & 3], b[(k + 1) & 3], acc[k], 0, 0, 0);
    }
    float s = 0.f;
#pragma unroll
    for (int k = 0; k < 12; ++k)
#pragma unroll
        for (int j = 0; j < 16; ++j) s += acc[k][j];
    out[blockIdx.x * 256 + threadIdx.x] = s;
}

// fp32 operands: zeros or the same pattern, scaled down so that the accumulators stay finite over the loop
__global__ void __launch_bounds__(256) mfma_fill_f32_kernel(float* __restrict__ in, int random_operands) {
    const int i = blockIdx.x * 256 + threadIdx.x;
    uint32_t x = (uint32_t)i * 1664525u + 1013904223u;
    x ^= x >> 15; x *= 2246822519u; x ^= x >> 13;
    in[i] = random_operands ? ((int)(x % 4001u) - 2000) / 1000.f : 0.f;
}

// bf16 operands: zeros, or a fixed pseudo-random pattern of values in (-2, 2) (an LCG over the piece index)
__global__ void __launch_bounds__(256) mfma_fill_kernel(uint16_t* __restrict__ in, int random_operands) {
    const int i = blockIdx.x * 256 + threadIdx.x;
    uint32_t x = (uint32_t)i * 1664525u + 1013904223u;
    x ^= x >> 15; x *= 2246822519u; x ^= x >> 13;
    const float f = ((int)(x % 4001u) - 2000) / 1000.f;
    in[i] = random_operands ? (uint16_t)(__float_as_uint(f) >> 16) : (uint16_t)0;
}

}  // namespace

extern "C" {

// Enqueues the loop (one workgroup of four waves per CU, 12 x iters MFMA instructions per wave) on `stream` and stores
// in *flop the floating point operations it performs; the caller times the stream.  random_operands = 0: all-zero
// operands; 1: a fixed pseudo-random pattern in (-2, 2).  ws: device scratch of bench_probe_mfma_workspace_bytes()
// bytes, 16-byte aligned.  Returns 0, -1 (bad argument), -3 (scratch too small) or -4 (launch failed).
size_t bench_probe_mfma_workspace_bytes(void) { return 65536 + 1024 * 256 * sizeof(float); }

int bench_probe_mfma(int random_operands, int iters, void* ws, size_t ws_bytes, double* flop, void* stream) {
    if (!ws || !flop || iters <= 0 || ((uintptr_t)ws & 15)) return -1;
    if (ws_bytes < bench_probe_mfma_workspace_bytes()) return -3;
    int dev = 0, cus = 256;
    if (hipGetDevice(&dev) == hipSuccess) (void)hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev);
    if (cus > 1024) cus = 1024;
    mfma_fill_kernel<<<128, 256, 0, (hipStream_t)stream>>>((uint16_t*)ws, random_operands ? 1 : 0);
    if (hipGetLastError() != hipSuccess) return -4;
    mfma_rate_kernel<<<cus, 256, 0, (hipStream_t)stream>>>((const uint4*)ws, (float*)((char*)ws + 65536), iters);
    *flop = 2.0 * 32 * 32 * 16 * 12.0 * (double)iters * 4.0 * cus;
    return hipGetLastError() == hipSuccess ? 0 : -4;
}

// The fp32 loop (v_mfma_f32_32x32x2_f32), same arguments and return codes.
int bench_probe_mfma_f32(int random_operands, int iters, void* ws, size_t ws_bytes, double* flop, void* stream) {
    if (!ws || !flop || iters <= 0 || ((uintptr_t)ws & 15)) return -1;
    if (ws_bytes < bench_probe_mfma_workspace_bytes()) return -3;
    int dev = 0, cus = 256;
    if (hipGetDevice(&dev) == hipSuccess) (void)hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev);
    if (cus > 1024) cus = 1024;
    mfma_fill_f32_kernel<<<64, 256, 0, (hipStream_t)stream>>>((float*)ws, random_operands ? 1 : 0);   // 16384 floats = 64 KB
    if (hipGetLastError() != hipSuccess) return -4;
    mfma_rate_f32_kernel<<<cus, 256, 0, (hipStream_t)stream>>>((const float*)ws, (float*)((char*)ws + 65536), iters);
    *flop = 2.0 * 32 * 32 * 2 * 12.0 * (double)iters * 4.0 * cus;
    return hipGetLastError() == hipSuccess ? 0 : -4;
}

}  // extern "C"
