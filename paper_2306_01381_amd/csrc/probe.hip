// Measurement aids (include/adaqp_probe.h): plain streams of a given size, the yardstick for the codec kernels.
// Nothing here is part of the method.
#include "common.hpp"
#include "adaqp_probe.h"

namespace adaqp {
namespace {

typedef float float4_t __attribute__((ext_vector_type(4)));

// Wave w reads K consecutive KiB (instruction j: 1 KiB) and writes K * 128 bytes.
template <int K>
__global__ __launch_bounds__(kBlock) void stream_read_kernel(const float *src, int64_t n_vec, uint32_t *dst)
{
    const int lane = threadIdx.x & (kWave - 1);
    const int64_t w = (int64_t)blockIdx.x * kWavesPerBlock + (threadIdx.x >> 6);
    const int64_t base = w * (kWave * K);
    float4_t x[K];
#pragma unroll
    for (int j = 0; j < K; ++j) {
        int64_t i = base + j * kWave + lane;
        i = i < n_vec ? i : n_vec - 1;
        x[j] = __builtin_nontemporal_load(reinterpret_cast<const float4_t *>(src) + i);
    }
#pragma unroll
    for (int j = 0; j + 1 < K; j += 2) {
        const uint32_t word = __builtin_bit_cast(uint32_t, x[j][0]) ^ __builtin_bit_cast(uint32_t, x[j + 1][3]);
        if (base + j * kWave + lane < n_vec) dst[w * (kWave * (K / 2)) + (j / 2) * kWave + lane] = word;
    }
}

// Wave w writes K consecutive KiB and reads K * 128 bytes.
template <int K>
__global__ __launch_bounds__(kBlock) void stream_write_kernel(const uint32_t *src, int64_t n_vec, float *dst)
{
    const int lane = threadIdx.x & (kWave - 1);
    const int64_t w = (int64_t)blockIdx.x * kWavesPerBlock + (threadIdx.x >> 6);
    const int64_t base = w * (kWave * K);
    uint32_t q[K / 2];
#pragma unroll
    for (int j = 0; j < K / 2; ++j) q[j] = src[w * (kWave * (K / 2)) + j * kWave + lane];
#pragma unroll
    for (int j = 0; j < K; ++j) {
        const int64_t i = base + j * kWave + lane;
        const float f = (float)(q[j / 2] >> (16 * (j & 1)));
        const float4_t v = {f, f + 1.0f, f + 2.0f, f + 3.0f};
        if (i < n_vec) __builtin_nontemporal_store(v, reinterpret_cast<float4_t *>(dst) + i);
    }
}

// Wave w reads K consecutive KiB of dst and K * 128 bytes of src, and writes the K KiB back.
template <int K>
__global__ __launch_bounds__(kBlock) void stream_update_kernel(const uint32_t *src, int64_t n_vec, float *dst)
{
    const int lane = threadIdx.x & (kWave - 1);
    const int64_t w = (int64_t)blockIdx.x * kWavesPerBlock + (threadIdx.x >> 6);
    const int64_t base = w * (kWave * K);
    uint32_t q[K / 2];
    float4_t x[K];
#pragma unroll
    for (int j = 0; j < K; ++j) {
        int64_t i = base + j * kWave + lane;
        i = i < n_vec ? i : n_vec - 1;
        x[j] = __builtin_nontemporal_load(reinterpret_cast<const float4_t *>(dst) + i);
    }
#pragma unroll
    for (int j = 0; j < K / 2; ++j) q[j] = src[w * (kWave * (K / 2)) + j * kWave + lane];
#pragma unroll
    for (int j = 0; j < K; ++j) {
        const int64_t i = base + j * kWave + lane;
        x[j][0] = __builtin_bit_cast(float, __builtin_bit_cast(uint32_t, x[j][0]) ^ (q[j / 2] >> (16 * (j & 1))));
        if (i < n_vec) __builtin_nontemporal_store(x[j], reinterpret_cast<float4_t *>(dst) + i);
    }
}

// Which XCD each workgroup of a 1-D grid runs on (hardware register XCC_ID).
__global__ __launch_bounds__(kBlock) void xcd_of_workgroup_kernel(int32_t *out, int32_t n)
{
    uint32_t xcc;
    asm volatile("s_getreg_b32 %0, hwreg(HW_REG_XCC_ID)" : "=s"(xcc));
    if (threadIdx.x == 0 && (int32_t)blockIdx.x < n) out[blockIdx.x] = (int32_t)(xcc & 0xF);
}

}  // namespace
}  // namespace adaqp

using namespace adaqp;

extern "C" int adaqp_probe_xcd_of_workgroup(int32_t *xcd_out_dev, int32_t n_workgroups, void *stream)
{
    if (n_workgroups < 0) return ADAQP_EINVAL;
    if (n_workgroups == 0) return ADAQP_OK;
    if (!xcd_out_dev || !aligned_to(xcd_out_dev, 4)) return ADAQP_EINVAL;
    hipLaunchKernelGGL(xcd_of_workgroup_kernel, dim3((unsigned)n_workgroups), dim3(kBlock), 0, (hipStream_t)stream,
                       xcd_out_dev, n_workgroups);
    ADAQP_HIP_TRY(hipGetLastError());
    return ADAQP_OK;
}

extern "C" int adaqp_probe_stream(const void *src_dev, void *dst_dev, int64_t bytes, int32_t write_side, void *stream)
{
    if (bytes < 0 || (bytes & 15) != 0) return ADAQP_EINVAL;
    if (bytes == 0) return ADAQP_OK;
    if (!src_dev || !dst_dev || !aligned_to(src_dev, 16) || !aligned_to(dst_dev, 16)) return ADAQP_EINVAL;
    if (bytes > ((int64_t)1 << 40)) return ADAQP_ESIZE;
    const int64_t n_vec = bytes / 16;
    hipStream_t st = (hipStream_t)stream;
    if (write_side < 0 || write_side > 2) return ADAQP_EINVAL;
    if (write_side == 2) {
        constexpr int K = 4;
        const int64_t waves = (n_vec + kWave * K - 1) / (kWave * K);
        const int64_t blocks = (waves + kWavesPerBlock - 1) / kWavesPerBlock;
        hipLaunchKernelGGL(stream_update_kernel<K>, dim3((unsigned)blocks), dim3(kBlock), 0, st,
                           static_cast<const uint32_t *>(src_dev), n_vec, static_cast<float *>(dst_dev));
    } else if (write_side) {
        constexpr int K = 4;
        const int64_t waves = (n_vec + kWave * K - 1) / (kWave * K);
        const int64_t blocks = (waves + kWavesPerBlock - 1) / kWavesPerBlock;
        hipLaunchKernelGGL(stream_write_kernel<K>, dim3((unsigned)blocks), dim3(kBlock), 0, st,
                           static_cast<const uint32_t *>(src_dev), n_vec, static_cast<float *>(dst_dev));
    } else {
        constexpr int K = 2;
        const int64_t waves = (n_vec + kWave * K - 1) / (kWave * K);
        const int64_t blocks = (waves + kWavesPerBlock - 1) / kWavesPerBlock;
        hipLaunchKernelGGL(stream_read_kernel<K>, dim3((unsigned)blocks), dim3(kBlock), 0, st,
                           static_cast<const float *>(src_dev), n_vec, static_cast<uint32_t *>(dst_dev));
    }
    ADAQP_HIP_TRY(hipGetLastError());
    return ADAQP_OK;
}
