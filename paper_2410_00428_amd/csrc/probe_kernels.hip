// Measurement helper: what the matrix cores of this GPU sustain on a stream of bf16 MFMAs with
// non-trivial operands, and at which shader clock.  The published dense peak assumes the boost clock; under
// a sustained matrix load the clock settles lower, and how far depends on the operand bits.  bench.py prints
// this figure next to the prefill attention rate so the two can be compared on the same box and minute.
#include <chrono>

#include "lkv_internal.hpp"

namespace {

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

// bf16 pairs with random sign and mantissa and exponents around 2^-4 .. 2^-1 (magnitudes of the workloads' data)
__device__ __forceinline__ unsigned random_bf16_pair(unsigned x) {
  x *= 2654435761u;
  x ^= x >> 15;
  x *= 2246822519u;
  x ^= x >> 13;
  return (x & 0x807f807fu) | 0x3d003d00u | ((x >> 3) & 0x03000300u);
}

// Every wavefront issues four independent chains of v_mfma_f32_32x32x16_bf16; nothing else is in the loop.
__global__ void __launch_bounds__(256) mfma_stream_kernel(float *sink, long long *clocks, int iters, int random_operands) {
  const int tid = threadIdx.x;
  const long long c0 = __builtin_readcyclecounter(), r0 = __builtin_amdgcn_s_memrealtime();
  u32x4 a[4], b;
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int w = 0; w < 4; ++w)
      a[i][w] = random_operands ? random_bf16_pair((blockIdx.x * 256u + tid) * 16u + i * 4 + w) : 0x3f803f80u;
#pragma unroll
  for (int w = 0; w < 4; ++w) b[w] = random_operands ? random_bf16_pair(0x9e3779b9u + tid * 4 + w) : 0x3f803f80u;
  f32x16 acc[4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[i][v] = 0.f;
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int i = 0; i < 4; ++i)
      acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a[i]), __builtin_bit_cast(bf16x8, b),
                                                       acc[i], 0, 0, 0);
  }
  float s = 0.f;
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int v = 0; v < 16; ++v) s += acc[i][v];
  if (s == 123.456f) sink[0] = s;  // keeps the accumulators alive
  if (tid == 0 && blockIdx.x % 8 == 0) {
    clocks[2 * (blockIdx.x / 8)] = __builtin_readcyclecounter() - c0;
    clocks[2 * (blockIdx.x / 8) + 1] = __builtin_amdgcn_s_memrealtime() - r0;
  }
}

// One wavefront writes n pairs (constant-rate clock, shader cycle counter), about `gap` shader cycles apart, and
// exits: next to another stream's work it shows what the shader clock does under that load.  Every wait is bounded.
__global__ void __launch_bounds__(64) clock_trace_kernel(long long *out, int n, int gap) {
  if (threadIdx.x != 0) return;
  for (int i = 0; i < n; ++i) {
    out[2 * i] = __builtin_amdgcn_s_memrealtime();
    out[2 * i + 1] = __builtin_readcyclecounter();
    const long long c0 = __builtin_readcyclecounter();
    for (int guard = 0; guard < 100000 && __builtin_readcyclecounter() - c0 < gap; ++guard) __builtin_amdgcn_s_sleep(64);
  }
}

}  // namespace

namespace lkv {

hipError_t probe_clock_trace(long long *out_dev, int n, int gap_cycles, int *wall_khz, hipStream_t s) {
  int dev = 0;
  hipError_t e;
  if ((e = hipGetDevice(&dev)) != hipSuccess) return e;
  if ((e = hipDeviceGetAttribute(wall_khz, hipDeviceAttributeWallClockRate, dev)) != hipSuccess) return e;
  hipLaunchKernelGGL(clock_trace_kernel, dim3(1), dim3(64), 0, s, out_dev, n, gap_cycles);
  return hipGetLastError();
}

hipError_t probe_mfma_rate(double millis, int random_operands, double *tflops, double *clock_mhz, hipStream_t s) {
  int cus = 0, wall_khz = 0;
  hipError_t e;
  if ((e = hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, 0)) != hipSuccess) return e;
  int dev = 0;
  if ((e = hipGetDevice(&dev)) != hipSuccess) return e;
  if ((e = hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev)) != hipSuccess) return e;
  if ((e = hipDeviceGetAttribute(&wall_khz, hipDeviceAttributeWallClockRate, dev)) != hipSuccess) return e;
  const int blocks = 2 * cus;  // two wavefronts per SIMD, as in the attention kernel
  float *sink = nullptr;
  long long *clocks = nullptr;
  if ((e = hipMalloc(&sink, 64)) != hipSuccess) return e;
  if ((e = hipMalloc(&clocks, (size_t)blocks / 8 * 16 + 16)) != hipSuccess) {
    (void)hipFree(sink);
    return e;
  }
  hipEvent_t a, b;
  (void)hipEventCreate(&a);
  (void)hipEventCreate(&b);
  auto run = [&](int iters, float *ms) -> hipError_t {
    hipError_t r = hipMemsetAsync(clocks, 0, (size_t)blocks / 8 * 16 + 16, s);
    if (r != hipSuccess) return r;
    (void)hipEventRecord(a, s);
    hipLaunchKernelGGL(mfma_stream_kernel, dim3(blocks), dim3(256), 0, s, sink, clocks, iters, random_operands);
    (void)hipEventRecord(b, s);
    if ((r = hipEventSynchronize(b)) != hipSuccess) return r;
    return hipEventElapsedTime(ms, a, b);
  };
  float ms = 0.f;
  const int cal_iters = 20000;  // ~1 ms
  e = run(cal_iters, &ms);
  if (e == hipSuccess) {
    double want = millis > 0 ? millis : 10.0;
    if (want > 200.0) want = 200.0;
    const int iters = (int)(cal_iters * want / (ms > 0.05f ? ms : 0.05f));
    e = run(iters > cal_iters ? iters : cal_iters, &ms);
    if (e == hipSuccess) {
      const int used = iters > cal_iters ? iters : cal_iters;
      const double flops = 2.0 * 32 * 32 * 16 * 4.0 * used * 4.0 * blocks;
      *tflops = flops / (ms * 1e-3) / 1e12;
      std::vector<long long> h((size_t)blocks / 8 * 2 + 2);
      e = hipMemcpy(h.data(), clocks, h.size() * 8, hipMemcpyDeviceToHost);
      double sc = 0, sr = 0;
      for (int i = 0; i < blocks / 8; ++i)
        if (h[2 * i + 1] > 0) {
          sc += (double)h[2 * i];
          sr += (double)h[2 * i + 1];
        }
      *clock_mhz = sr > 0 ? sc / sr * (wall_khz / 1000.0) : 0.0;
    }
  }
  (void)hipEventDestroy(a);
  (void)hipEventDestroy(b);
  (void)hipFree(sink);
  (void)hipFree(clocks);
  return e;
}

}  // namespace lkv
