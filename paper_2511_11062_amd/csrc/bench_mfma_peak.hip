// Benchmark-only diagnostic, built into its own shared object (libla_bench_mfma.so) and loaded by bench.py alone:
// a register-resident loop of v_mfma_f32_32x32x16_bf16 with no memory traffic.  The sustained matrix-core clock
// depends on the operands' bit patterns (power), so the rate of this loop on the workload's own data is the practical
// ceiling of the fused attention kernel on that data.  Nothing in the attention library links or calls this file.
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

// 8 A and 8 B fragments per lane read once from `data`, then iters x 32 MFMAs on four independent accumulators.
__global__ __launch_bounds__(256, 2) void mfma_peak_kernel(const uint4* __restrict__ data, float* __restrict__ sink,
                                                            int iters) {
  bf16x8 a[8], b[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    const uint4 x = data[(threadIdx.x + 256 * i) & 4095], y = data[(threadIdx.x + 256 * i + 2048) & 4095];
    a[i] = __builtin_bit_cast(bf16x8, x);
    b[i] = __builtin_bit_cast(bf16x8, y);
  }
  f32x16 acc[4];
#pragma unroll
  for (int n = 0; n < 4; ++n)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[n][r] = 0.f;
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int u = 0; u < 32; ++u)
      acc[u & 3] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[u & 7], b[(u >> 2) & 7], acc[u & 3], 0, 0, 0);
  }
  float s = 0.f;
#pragma unroll
  for (int n = 0; n < 4; ++n)
#pragma unroll
    for (int r = 0; r < 16; ++r) s += acc[n][r];
  if (s == 12345.678f) sink[0] = s;  // keeps the loop alive without a store in the common case
}

}  // namespace

// Times `iters` x 32 MFMAs per wave, 2 waves per SIMD on every CU, operands taken from `dev_operands` (device
// pointer, at least 64 KiB, read as bf16), on `hip_stream`; synchronises.  Returns 0 or the hipError_t that failed;
// on success *host_ms is the elapsed time and *host_flops the flop count.
extern "C" int la_bench_mfma_peak(void* hip_stream, const void* dev_operands, int iters, float* host_ms,
                                  double* host_flops) {
  if (!dev_operands || !host_ms || !host_flops || iters < 1 || iters > (1 << 20)) return (int)hipErrorInvalidValue;
  hipStream_t st = reinterpret_cast<hipStream_t>(hip_stream);
  int dev = 0, cus = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e == hipSuccess) e = hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev);
  if (e != hipSuccess) return (int)e;
  const int blocks = 2 * cus;  // 2 workgroups of 4 waves per CU: 2 waves per SIMD
  float* sink = nullptr;
  hipEvent_t e0 = nullptr, e1 = nullptr;
  e = hipMalloc(&sink, sizeof(float));
  if (e == hipSuccess) e = hipEventCreate(&e0);
  if (e == hipSuccess) e = hipEventCreate(&e1);
  const uint4* data = static_cast<const uint4*>(dev_operands);
  if (e == hipSuccess) {
    hipLaunchKernelGGL(mfma_peak_kernel, dim3(blocks), dim3(256), 0, st, data, sink, 64);  // warm-up
    e = hipGetLastError();
  }
  if (e == hipSuccess) e = hipEventRecord(e0, st);
  if (e == hipSuccess) {
    hipLaunchKernelGGL(mfma_peak_kernel, dim3(blocks), dim3(256), 0, st, data, sink, iters);
    e = hipGetLastError();
  }
  if (e == hipSuccess) e = hipEventRecord(e1, st);
  if (e == hipSuccess) e = hipEventSynchronize(e1);
  if (e == hipSuccess) e = hipEventElapsedTime(host_ms, e0, e1);
  if (e0) (void)hipEventDestroy(e0);
  if (e1) (void)hipEventDestroy(e1);
  if (sink) (void)hipFree(sink);
  if (e != hipSuccess) return (int)e;
  *host_flops = (double)blocks * 4.0 * (double)iters * 32.0 * (2.0 * 32 * 32 * 16);
  return 0;
}
