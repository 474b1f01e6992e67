// Calibration of the smoothing factors (Eq. 4): lambda_i = sqrt(max over the calibration tokens of |K[., i]|),
// per KV head and channel.  |x| of an fp16 value is exact and a non-negative fp32 orders like its
// bit pattern, so the maximum is taken with integer atomics directly in the output array and is
// the same whatever the order; a last pass takes the square root in place.
#include "common.h"

namespace vecinfer {

namespace {

constexpr int kCalBlock = 256;
constexpr int kCalTokens = 256;     // tokens per workgroup

__global__ void lambda_zero_kernel(float *lam, int n)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) lam[i] = 0.f;
}

// grid (token chunks, Hkv, B); a thread owns one channel (D <= 128 < kCalBlock: the block holds
// kCalBlock / D token lanes per channel)
__global__ __launch_bounds__(kCalBlock) void lambda_max_kernel(const __half *k, float *lam, int Hkv, int D, long long T)
{
    const int c = threadIdx.x % D, lane_t = threadIdx.x / D, per = kCalBlock / D;
    const int g = blockIdx.y, b = blockIdx.z;
    const long long t0 = (long long)blockIdx.x * kCalTokens;
    const long long t1 = t0 + kCalTokens < T ? t0 + kCalTokens : T;
    const __half *row = k + ((size_t)b * Hkv + g) * T * D;
    float mx = 0.f;
    for (long long t = t0 + lane_t; t < t1; t += per) mx = fmaxf(mx, fabsf(__half2float(row[t * D + c])));
    atomicMax(reinterpret_cast<unsigned *>(lam) + (size_t)g * D + c, __float_as_uint(mx));
}

__global__ void lambda_finalize_kernel(float *lam, int n, float floor_value)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) lam[i] = fmaxf(sqrtf(lam[i]), floor_value);
}

} // namespace

int launch_calibrate_lambda(const __half *k, float *lam, int B, int Hkv, int D, long long T, float floor_value,
                            hipStream_t stream)
{
    const int n = Hkv * D;
    hipLaunchKernelGGL(lambda_zero_kernel, dim3((n + 255) / 256), dim3(256), 0, stream, lam, n);
    if (hipGetLastError() != hipSuccess) return -4;
    dim3 grid((unsigned)((T + kCalTokens - 1) / kCalTokens), Hkv, B);
    hipLaunchKernelGGL(lambda_max_kernel, grid, dim3(kCalBlock), 0, stream, k, lam, Hkv, D, T);
    if (hipGetLastError() != hipSuccess) return -4;
    hipLaunchKernelGGL(lambda_finalize_kernel, dim3((n + 255) / 256), dim3(256), 0, stream, lam, n, floor_value);
    return hipGetLastError() == hipSuccess ? 0 : -4;
}

} // namespace vecinfer
