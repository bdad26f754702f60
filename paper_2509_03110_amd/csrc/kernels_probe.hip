// Ceilings of the chip measured with the simplest possible kernels, for reading the roofline
// fractions against: a plain device copy and loops of nothing but independent MFMAs.
#include "engine.h"

namespace lsam {
namespace {

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

__global__ __launch_bounds__(256) void probe_copy_kernel(const f32x4* __restrict__ src,
                                                         f32x4* __restrict__ dst, long long n) {
  const long long i = (long long)blockIdx.x * 256 + threadIdx.x;
  if (i < n) __builtin_nontemporal_store(__builtin_nontemporal_load(src + i), dst + i);
}

// Four wavefronts per workgroup, each issuing `iters` rounds of 8 MFMAs on 8 independent
// accumulators with operands that never leave registers.
template <bool BF16>
__global__ __launch_bounds__(256) void probe_mfma_kernel(float* __restrict__ sink, int iters) {
  f32x16 acc[8];
#pragma unroll
  for (int a = 0; a < 8; ++a)
#pragma unroll
    for (int e = 0; e < 16; ++e) acc[a][e] = 0.f;
  const float seed = (float)(threadIdx.x & 7) * 0.125f;
  bf16x8 xa, xb;
#pragma unroll
  for (int e = 0; e < 8; ++e) { xa[e] = static_cast<__bf16>(seed); xb[e] = static_cast<__bf16>(1.f - seed); }
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int a = 0; a < 8; ++a) {
      if constexpr (BF16) acc[a] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(xa, xb, acc[a], 0, 0, 0);
      else acc[a] = __builtin_amdgcn_mfma_f32_32x32x2f32(seed, 1.f - seed, acc[a], 0, 0, 0);
    }
  }
  float s = 0.f;
#pragma unroll
  for (int a = 0; a < 8; ++a)
#pragma unroll
    for (int e = 0; e < 16; ++e) s += acc[a][e];
  if (s == 12345.678f) sink[0] = s;      // keeps the loop alive without a store in practice
}

}  // namespace

// Times `launch` between two events on `s`, best of `reps`; milliseconds, < 0 on error.
template <typename F>
static float best_ms(hipStream_t s, int reps, F launch) {
  hipEvent_t a = nullptr, b = nullptr;
  if (hipEventCreate(&a) != hipSuccess || hipEventCreate(&b) != hipSuccess) return -1.f;
  float best = -1.f;
  for (int r = 0; r < reps; ++r) {
    if (hipEventRecord(a, s) != hipSuccess) break;
    launch();
    if (hipEventRecord(b, s) != hipSuccess || hipEventSynchronize(b) != hipSuccess) break;
    float ms = 0.f;
    if (hipEventElapsedTime(&ms, a, b) != hipSuccess) break;
    if (best < 0.f || ms < best) best = ms;
  }
  (void)hipEventDestroy(a);
  (void)hipEventDestroy(b);
  return best;
}

int probe_peaks(void* scratch, size_t bytes, hipStream_t s, double* copy_gbs, double* bf16_tflops,
                double* f32_tflops) {
  const long long half = (long long)(bytes / 2 / 16);            // 16-byte words per half
  if (half < 1024 || (reinterpret_cast<uintptr_t>(scratch) & 15)) return -1;
  const f32x4* src = static_cast<const f32x4*>(scratch);
  f32x4* dst = static_cast<f32x4*>(scratch) + half;
  const unsigned blocks = (unsigned)((half + 255) / 256);
  float ms = best_ms(s, 4, [&] { probe_copy_kernel<<<blocks, 256, 0, s>>>(src, dst, half); });
  if (ms <= 0.f) return -1;
  *copy_gbs = 2.0 * (double)half * 16.0 / (ms * 1e-3) / 1e9;     // bytes read + bytes written
  int dev = 0, cus = 0;
  if (hipGetDevice(&dev) != hipSuccess ||
      hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess)
    return -1;
  const int grid = cus * 2, iters = 4096;
  float* sink = static_cast<float*>(scratch);
  ms = best_ms(s, 3, [&] { probe_mfma_kernel<true><<<grid, 256, 0, s>>>(sink, iters); });
  if (ms <= 0.f) return -1;
  *bf16_tflops = (double)grid * 4 * iters * 8 * (2.0 * 32 * 32 * 16) / (ms * 1e-3) / 1e12;
  ms = best_ms(s, 3, [&] { probe_mfma_kernel<false><<<grid, 256, 0, s>>>(sink, iters / 2); });
  if (ms <= 0.f) return -1;
  *f32_tflops = (double)grid * 4 * (iters / 2) * 8 * (2.0 * 32 * 32 * 2) / (ms * 1e-3) / 1e12;
  return hipGetLastError() == hipSuccess ? 0 : -1;
}

}  // namespace lsam
