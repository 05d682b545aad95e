// Hessian-based sensitivity (Sec. 3.2): the power iteration of Alg. 1 as a stream of kernels around a caller's
// Hessian-vector product, and Eq. 2 on the host.
//
// The iteration never comes back to the host: the norm and the eigenvalue estimate of a step are reduced on the
// device (two stages, fixed order: the result does not depend on scheduling), the next vector is scaled by a
// kernel that reads the norm from device memory, and the estimates of all steps are left in a device array.
#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdint>
#include <vector>

#include "qb_common.hpp"

namespace qb {
namespace {

constexpr int PI_BLOCKS = 256;  // partial sums per reduction

// part[b] = sum over block b's grid-stride share of a*b, part[PI_BLOCKS + b] = the same of b*b
__global__ __launch_bounds__(256) void pi_partial_kernel(const float *__restrict__ a, const float *__restrict__ b,
                                                         int64_t n, float *__restrict__ part)
{
    __shared__ float red[8];
    float sab = 0.0f, sbb = 0.0f;
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (int64_t)gridDim.x * 256) {
        const float x = a[i], y = b[i];
        sab += x * y;
        sbb += y * y;
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
        sab += __shfl_xor(sab, o);
        sbb += __shfl_xor(sbb, o);
    }
    if ((threadIdx.x & 63) == 0) {
        red[threadIdx.x >> 6] = sab;
        red[4 + (threadIdx.x >> 6)] = sbb;
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        part[blockIdx.x] = (red[0] + red[1]) + (red[2] + red[3]);
        part[PI_BLOCKS + blockIdx.x] = (red[4] + red[5]) + (red[6] + red[7]);
    }
}

// one wavefront: the partial sums in a fixed order -> fin[0] = a.b, fin[1] = |b|; optionally the step's estimate
__global__ __launch_bounds__(64) void pi_finish_kernel(const float *__restrict__ part, int blocks, float *__restrict__ fin,
                                                       float *__restrict__ estimate)
{
    float sab = 0.0f, sbb = 0.0f;
    for (int i = threadIdx.x; i < blocks; i += 64) {
        sab += part[i];
        sbb += part[PI_BLOCKS + i];
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
        sab += __shfl_xor(sab, o);
        sbb += __shfl_xor(sbb, o);
    }
    if (threadIdx.x == 0) {
        fin[0] = sab;
        fin[1] = sqrtf(sbb);
        if (estimate) *estimate = sab;
    }
}

// v = src / |src| with the norm read from device memory; a zero vector is left as zeros (src may be v itself)
__global__ __launch_bounds__(256) void pi_scale_kernel(const float *src, int64_t n, const float *__restrict__ fin, float *v)
{
    const float nrm = fin[1];
    const float inv = nrm > 0.0f ? 1.0f / nrm : 0.0f;
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (int64_t)gridDim.x * 256) v[i] = src[i] * inv;
}

}  // namespace
}  // namespace qb

using namespace qb;

extern "C" size_t qb_power_iteration_scratch_floats(void) { return 2 * PI_BLOCKS + 2; }

extern "C" qb_status qb_power_iteration(qb_hv_fn hv, void *ctx, int64_t n, int iters, float *v, float *hv_buf,
                                        float *scratch, float *estimates, void *stream)
{
    if (!hv || !v || !hv_buf || !scratch || !estimates) return QB_ERR_NULL;
    if (n <= 0 || iters <= 0) return QB_ERR_SHAPE;
    hipStream_t st = static_cast<hipStream_t>(stream);
    int blocks = (int)((n + 1023) / 1024);
    if (blocks > PI_BLOCKS) blocks = PI_BLOCKS;
    if (blocks < 1) blocks = 1;
    float *part = scratch, *fin = scratch + 2 * PI_BLOCKS;
    // v = v / |v|
    hipLaunchKernelGGL(pi_partial_kernel, dim3(blocks), dim3(256), 0, st, v, v, n, part);
    hipLaunchKernelGGL(pi_finish_kernel, dim3(1), dim3(64), 0, st, part, blocks, fin, static_cast<float *>(nullptr));
    hipLaunchKernelGGL(pi_scale_kernel, dim3(blocks), dim3(256), 0, st, v, n, fin, v);
    for (int i = 0; i < iters; ++i) {
        if (hv(ctx, v, hv_buf, stream) != 0) return QB_ERR_HIP;
        hipLaunchKernelGGL(pi_partial_kernel, dim3(blocks), dim3(256), 0, st, v, hv_buf, n, part);
        hipLaunchKernelGGL(pi_finish_kernel, dim3(1), dim3(64), 0, st, part, blocks, fin, estimates + i);
        hipLaunchKernelGGL(pi_scale_kernel, dim3(blocks), dim3(256), 0, st, hv_buf, n, fin, v);
    }
    return launch_status();
}

extern "C" qb_status qb_sensitivity_omega(const float *lambdas, int layers, int runs, float *omega)
{
    if (!lambdas || !omega) return QB_ERR_NULL;
    if (layers <= 0 || runs <= 0) return QB_ERR_SHAPE;
    for (int i = 0; i < layers; ++i) {
        double mean = 0.0, var = 0.0;
        for (int r = 0; r < runs; ++r) mean += (double)lambdas[(size_t)i * runs + r];
        mean /= runs;
        for (int r = 0; r < runs; ++r) {
            const double d = (double)lambdas[(size_t)i * runs + r] - mean;
            var += d * d;
        }
        omega[i] = (float)(std::fabs(mean) + std::sqrt(var / runs));
    }
    return QB_OK;
}

extern "C" qb_status qb_rank_by_sensitivity(const float *omega, int layers, int32_t *order)
{
    if (!omega || !order) return QB_ERR_NULL;
    if (layers <= 0) return QB_ERR_SHAPE;
    for (int i = 0; i < layers; ++i) order[i] = i;
    for (int i = 1; i < layers; ++i) {  // insertion sort: stable, and layers are few
        const int32_t k = order[i];
        int j = i - 1;
        while (j >= 0 && omega[order[j]] < omega[k]) {
            order[j + 1] = order[j];
            --j;
        }
        order[j + 1] = k;
    }
    return QB_OK;
}

// ---- measurement aid: the issue rate of the int8 matrix-core instruction the GEMM uses -------------------------
// Every wavefront runs `iters` rounds of four independent v_mfma_i32_32x32x32_i8 on registers, nothing else:
// 4 * 65536 integer operations per round and wavefront.  Timed by the caller (events around the launch).
namespace qb {
namespace {
typedef int pv4i __attribute__((ext_vector_type(4)));
typedef int pv16i __attribute__((ext_vector_type(16)));
__global__ __launch_bounds__(256) void mfma_i8_probe_kernel(int iters, int32_t *sink)
{
    const int lane = threadIdx.x & 63;
    const pv4i a = {lane, lane + 1, lane + 2, lane + 3}, b = {1, 2, 3, lane};
    pv16i c0 = {0}, c1 = {0}, c2 = {0}, c3 = {0};
    for (int i = 0; i < iters; ++i) {
        c0 = __builtin_amdgcn_mfma_i32_32x32x32_i8(a, b, c0, 0, 0, 0);
        c1 = __builtin_amdgcn_mfma_i32_32x32x32_i8(a, b, c1, 0, 0, 0);
        c2 = __builtin_amdgcn_mfma_i32_32x32x32_i8(a, b, c2, 0, 0, 0);
        c3 = __builtin_amdgcn_mfma_i32_32x32x32_i8(a, b, c3, 0, 0, 0);
    }
    int s = 0;
#pragma unroll
    for (int i = 0; i < 16; ++i) s += c0[i] + c1[i] + c2[i] + c3[i];
    if (s == 0x7fffffff) sink[0] = s;  // keeps the loop alive; practically never taken
}
}  // namespace
}  // namespace qb

extern "C" qb_status qb_probe_mfma_i8(int workgroups, int iters, int32_t *sink, void *stream)
{
    if (!sink) return QB_ERR_NULL;
    if (workgroups <= 0 || workgroups > 65536 || iters <= 0) return QB_ERR_SHAPE;
    hipLaunchKernelGGL(mfma_i8_probe_kernel, dim3(workgroups), dim3(256), 0, static_cast<hipStream_t>(stream), iters, sink);
    return launch_status();
}
