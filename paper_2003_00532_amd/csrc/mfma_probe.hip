// libgemm_f64.so: the MFMA-only probe (declared in include/gemm_f64.h and include/gemm_f32.h).
//
// A register-resident loop of independent matrix instructions with no memory traffic: what the matrix
// pipes sustain at the clock the chip actually holds, to be reported beside the published peak.
#include "../../include/gemm_f32.h"

#include <hip/hip_runtime.h>

#include "gemm_mfma.hpp"

using namespace gemm_detail;

namespace {

int current_probe_cus()
{
    int dev = 0, v = 0;
    if (hipGetDevice(&dev) == hipSuccess &&
        hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && v > 0)
        return v;
    return 256;
}

constexpr int kProbeTiles = 16;          // independent accumulator tiles per wave
constexpr int kProbeWorkgroupsPerCu = 2;

template <typename T>
__global__ void __launch_bounds__(kThreads, 2) mfma_probe_kernel(int64_t iterations, T *__restrict__ sink)
{
    typedef Elem<T, 16> EL;
    typedef typename EL::acc_t acc_t;
    // operands small enough that the sums stay far from overflow for any iteration count in range
    const T a = T(1) / T(1 << 20) * T(1 + (threadIdx.x & 3)), b = T(1) / T(1 << 20);
    acc_t acc[kProbeTiles];
#pragma unroll
    for (int t = 0; t < kProbeTiles; ++t) acc[t] = acc_t{T(0), T(0), T(0), T(0)};
    for (int64_t it = 0; it < iterations; ++it) {
#pragma unroll
        for (int t = 0; t < kProbeTiles; ++t) acc[t] = EL::mfma(a, b, acc[t]);
    }
    T s = T(0);
#pragma unroll
    for (int t = 0; t < kProbeTiles; ++t) s += acc[t][0] + acc[t][1] + acc[t][2] + acc[t][3];
    sink[(int64_t)blockIdx.x * kThreads + threadIdx.x] = s;
}

template <typename T>
int probe(int64_t iterations, T *sink, int64_t sink_elems, void *stream, double *flops)
{
    if (iterations < 1 || iterations > ((int64_t)1 << 30)) return GEMM_F64_ERR_DIM;
    if (sink == nullptr) return GEMM_F64_ERR_NULL;
    const int64_t grid = (int64_t)current_probe_cus() * kProbeWorkgroupsPerCu;
    if (sink_elems < grid * kThreads) return GEMM_F64_ERR_DIM;
    hipLaunchKernelGGL(mfma_probe_kernel<T>, dim3((unsigned)grid), dim3(kThreads), 0, (hipStream_t)stream, iterations, sink);
    if (hipGetLastError() != hipSuccess) return GEMM_F64_ERR_LAUNCH;
    // every wave issues kProbeTiles MFMAs of 2 * 16 * 16 * 4 flop per iteration
    if (flops) *flops = (double)grid * (kThreads / 64) * (double)iterations * kProbeTiles * 2048.0;
    return GEMM_F64_OK;
}

}  // namespace

extern "C" int gemm_f64_mfma_probe(int64_t iterations, double *sink, int64_t sink_elems, void *stream, double *flops)
{
    return probe<double>(iterations, sink, sink_elems, stream, flops);
}

extern "C" int gemm_f32_mfma_probe(int64_t iterations, float *sink, int64_t sink_elems, void *stream, double *flops)
{
    return probe<float>(iterations, sink, sink_elems, stream, flops);
}

// The machine peak computed the way the paper computes its own (Section 1.2: units per core x width x clock):
// compute units x 4 SIMDs x flops of one 16x16x4 MFMA / its issue cycles (64 in double, 32 in float) x the
// clock the device reports.
extern "C" int gemm_f64_device_peak(int *compute_units, int *clock_khz, double *fp64_mfma_tflops, double *fp32_mfma_tflops)
{
    int dev = 0, cus = 0, khz = 0;
    if (hipGetDevice(&dev) != hipSuccess ||
        hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess ||
        hipDeviceGetAttribute(&khz, hipDeviceAttributeClockRate, dev) != hipSuccess || cus <= 0 || khz <= 0)
        return GEMM_F64_ERR_LAUNCH;
    if (compute_units) *compute_units = cus;
    if (clock_khz) *clock_khz = khz;
    const double mfma_flops = 2.0 * 16 * 16 * 4, hz = (double)khz * 1e3;
    if (fp64_mfma_tflops) *fp64_mfma_tflops = cus * 4 * (mfma_flops / 64.0) * hz / 1e12;
    if (fp32_mfma_tflops) *fp32_mfma_tflops = cus * 4 * (mfma_flops / 32.0) * hz / 1e12;
    return GEMM_F64_OK;
}
