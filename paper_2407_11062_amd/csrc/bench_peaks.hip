// Measurement aids for bench.py, built into their own library (libeqat_peaks.so), not part of libeqat.so:
// what this very chip, at the clocks it holds under this very load, gives (a) a loop of nothing but
// v_mfma_f32_32x32x16_bf16 or v_mfma_f32_16x16x32_bf16 (the GEMM kernels use both), (b) a plain device copy and (c) a kernel that only reads.  bench.py quotes every roofline fraction against the
// published peaks (2.5 PFLOP/s, 8 TB/s) and against these two.
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef unsigned int uintx4 __attribute__((ext_vector_type(4)));

constexpr int kWavesPerGroup = 8;      // two per SIMD, like the GEMM kernels
constexpr int kChains = 4;             // independent accumulators per wave: back-to-back issue without dependency stalls

// Every wave loads one A and one B fragment per chain from `data` (zeros, or random bf16: the power the chip draws,
// and with it the clock it holds, depends on the operand bits) and then runs iters * kChains MFMAs on them.
__global__ __launch_bounds__(64 * kWavesPerGroup) void k_mfma_loop(const uintx4 *__restrict__ data, uint32_t n_vec, int iters,
                                                                   float *__restrict__ sink)
{
    const uint32_t t = blockIdx.x * blockDim.x + threadIdx.x;
    bf16x8 a[kChains], b[kChains];
    floatx16 acc[kChains];
#pragma unroll
    for (int c = 0; c < kChains; ++c) {
        a[c] = __builtin_bit_cast(bf16x8, data[(t * 2 * kChains + 2 * c) % n_vec]);
        b[c] = __builtin_bit_cast(bf16x8, data[(t * 2 * kChains + 2 * c + 1) % n_vec]);
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[c][r] = 0.0f;
    }
    for (int i = 0; i < iters; ++i) {
#pragma unroll
        for (int c = 0; c < kChains; ++c) acc[c] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[c], b[c], acc[c], 0, 0, 0);
    }
    float s = 0.0f;
#pragma unroll
    for (int c = 0; c < kChains; ++c)
#pragma unroll
        for (int r = 0; r < 16; ++r) s += acc[c][r];
    if (s == 12345.678f) sink[0] = s;          // keeps the loop alive; practically never true
}

// The same with v_mfma_f32_16x16x32_bf16: half the flops per instruction, twice the instructions and chains.
constexpr int kChains16 = 8;
__global__ __launch_bounds__(64 * kWavesPerGroup) void k_mfma16_loop(const uintx4 *__restrict__ data, uint32_t n_vec, int iters,
                                                                     float *__restrict__ sink)
{
    const uint32_t t = blockIdx.x * blockDim.x + threadIdx.x;
    bf16x8 a[kChains16], b[kChains16];
    floatx4 acc[kChains16];
#pragma unroll
    for (int c = 0; c < kChains16; ++c) {
        a[c] = __builtin_bit_cast(bf16x8, data[(t * 2 * kChains16 + 2 * c) % n_vec]);
        b[c] = __builtin_bit_cast(bf16x8, data[(t * 2 * kChains16 + 2 * c + 1) % n_vec]);
#pragma unroll
        for (int r = 0; r < 4; ++r) acc[c][r] = 0.0f;
    }
    for (int i = 0; i < iters; ++i) {
#pragma unroll
        for (int c = 0; c < kChains16; ++c) acc[c] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[c], b[c], acc[c], 0, 0, 0);
    }
    float s = 0.0f;
#pragma unroll
    for (int c = 0; c < kChains16; ++c)
#pragma unroll
        for (int r = 0; r < 4; ++r) s += acc[c][r];
    if (s == 12345.678f) sink[0] = s;          // keeps the loop alive; practically never true
}

__global__ __launch_bounds__(256) void k_copy(const uintx4 *__restrict__ src, uintx4 *__restrict__ dst, size_t n_vec)
{
    size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    const size_t stride = (size_t)gridDim.x * 256;
    // four independent 16-byte loads in flight per lane
    for (; i + 3 * stride < n_vec; i += 4 * stride) {
        const uintx4 v0 = src[i], v1 = src[i + stride], v2 = src[i + 2 * stride], v3 = src[i + 3 * stride];
        dst[i] = v0; dst[i + stride] = v1; dst[i + 2 * stride] = v2; dst[i + 3 * stride] = v3;
    }
    for (; i < n_vec; i += stride) dst[i] = src[i];
}

// Reads `n_vec` 16-byte vectors once (eight loads in flight per lane) and keeps nothing: what a kernel that only has to
// fetch that many bytes can reach, launch and ramp-up included.
__global__ __launch_bounds__(256) void k_read(const uintx4 *__restrict__ src, size_t n_vec, uint32_t *__restrict__ sink)
{
    size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    const size_t stride = (size_t)gridDim.x * 256;
    uintx4 acc = {0u, 0u, 0u, 0u};
    for (; i + 7 * stride < n_vec; i += 8 * stride) {
        uintx4 v[8];
#pragma unroll
        for (int q = 0; q < 8; ++q) v[q] = src[i + q * stride];
#pragma unroll
        for (int q = 0; q < 8; ++q) acc ^= v[q];
    }
    for (; i < n_vec; i += stride) acc ^= src[i];
    if ((acc[0] ^ acc[1] ^ acc[2] ^ acc[3]) == 0x9E3779B9u) sink[0] = acc[0];      // keeps the loads alive; practically never true
}

}  // namespace

extern "C" {

// Flop of one launch of eqat_peak_mfma_loop: groups * 8 waves * iters * 4 MFMAs * 2 * 32 * 32 * 16.
double eqat_peak_mfma_flop(int groups, int iters) { return (double)groups * kWavesPerGroup * (double)iters * kChains * 32768.0; }

// data: device, data_bytes >= 16 and a multiple of 16; sink: one float, device.  Returns 0, or 1 on a bad argument / launch.
int eqat_peak_mfma_loop(const void *data, size_t data_bytes, int groups, int iters, float *sink, void *stream)
{
    if (data == nullptr || sink == nullptr || data_bytes < 16 || data_bytes % 16 != 0 || groups < 1 || iters < 1) return 1;
    k_mfma_loop<<<dim3(groups), dim3(64 * kWavesPerGroup), 0, (hipStream_t)stream>>>((const uintx4 *)data, (uint32_t)(data_bytes / 16),
                                                                                      iters, sink);
    return hipGetLastError() == hipSuccess ? 0 : 1;
}

// The 16x16x32 form: flop of one launch = groups * 8 waves * iters * 8 MFMAs * 2 * 16 * 16 * 32; arguments as above.
double eqat_peak_mfma16_flop(int groups, int iters) { return (double)groups * kWavesPerGroup * (double)iters * kChains16 * 16384.0; }
int eqat_peak_mfma16_loop(const void *data, size_t data_bytes, int groups, int iters, float *sink, void *stream)
{
    if (data == nullptr || sink == nullptr || data_bytes < 16 || data_bytes % 16 != 0 || groups < 1 || iters < 1) return 1;
    k_mfma16_loop<<<dim3(groups), dim3(64 * kWavesPerGroup), 0, (hipStream_t)stream>>>((const uintx4 *)data, (uint32_t)(data_bytes / 16),
                                                                                        iters, sink);
    return hipGetLastError() == hipSuccess ? 0 : 1;
}

// dst, src: device, 16-byte aligned, bytes a multiple of 16.
int eqat_peak_copy(void *dst, const void *src, size_t bytes, void *stream)
{
    if (dst == nullptr || src == nullptr || bytes % 16 != 0 || bytes == 0) return 1;
    k_copy<<<dim3(256 * 16), dim3(256), 0, (hipStream_t)stream>>>((const uintx4 *)src, (uintx4 *)dst, bytes / 16);
    return hipGetLastError() == hipSuccess ? 0 : 1;
}

// src: device, 16-byte aligned, bytes a multiple of 16; sink: one word, device.
int eqat_peak_read(const void *src, size_t bytes, void *sink, void *stream)
{
    if (src == nullptr || sink == nullptr || bytes % 16 != 0 || bytes == 0) return 1;
    const size_t n_vec = bytes / 16;
    size_t groups = (n_vec + 256 * 8 - 1) / (256 * 8);         // one trip of eight loads per lane, unless that needs too many workgroups
    if (groups > 256 * 16) groups = 256 * 16;
    k_read<<<dim3((unsigned)groups), dim3(256), 0, (hipStream_t)stream>>>((const uintx4 *)src, n_vec, (uint32_t *)sink);
    return hipGetLastError() == hipSuccess ? 0 : 1;
}

}  // extern "C"
