// Fused softmax cross-entropy forward + backward (one wavefront per sample row, wavefront
// shuffle reductions) and the bias gradient (column sums of dZ).
#include "engine.h"
#include "b32s.h"

namespace lsam {
namespace {

constexpr int kThreads = 256;
constexpr int kWaves = kThreads / 64;

__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) v = fmaxf(v, __shfl_xor(v, off, 64));
  return v;
}
__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
  return v;
}

template <typename TD>
__device__ __forceinline__ void put(TD* p, float v);
template <> __device__ __forceinline__ void put<float>(float* p, float v) { *p = v; }
template <> __device__ __forceinline__ void put<__bf16>(__bf16* p, float v) {
  *p = static_cast<__bf16>(v);
}

// Row r = replica*B + sample.  loss_row = logsumexp(z) - z[label];
// dz = (softmax(z) - onehot(label)) / B;  padded columns [C, ld_dz) are written as zero.
// TD = float: dz row-major with pitch ld_dz.  TD = bf16: dz in the blocked layout, one matrix
// [B][C] per replica, ld_dz = elements per replica (its padding is zero from initialisation).
template <typename TD>
__global__ __launch_bounds__(kThreads) void softmax_ce_kernel(
    const float* __restrict__ logits, int ld, const int32_t* __restrict__ labels,
    TD* __restrict__ dz, long long ld_dz, float* __restrict__ loss_rows, int rows, int B, int C) {
  const int lane = threadIdx.x & 63;
  const int r = blockIdx.x * kWaves + (threadIdx.x >> 6);
  if (r >= rows) return;
  const float* z = logits + (long long)r * ld;
  const int lab = labels[r];
  float mx = -INFINITY;
  for (int c = lane; c < C; c += 64) mx = fmaxf(mx, z[c]);
  mx = wave_max(mx);
  float se = 0.f;
  for (int c = lane; c < C; c += 64) se += __expf(z[c] - mx);
  se = wave_sum(se);
  const float inv = 1.f / se;
  const float invB = 1.f / (float)B;
  constexpr bool blocked = sizeof(TD) == 2;
  const int rep = r / B, b = r - rep * B;
  const int cb = b32s_blocks(C);
  const int width = blocked ? C : (int)ld_dz;
  for (int c = lane; c < width; c += 64) {
    float v = 0.f;
    if (c < C) {
      v = __expf(z[c] - mx) * inv;
      if (c == lab) v -= 1.f;
      v *= invB;
    }
    TD* d = blocked ? dz + (long long)rep * ld_dz + b32s_offset(b, c, cb) : dz + (long long)r * ld_dz + c;
    put<TD>(d, v);
  }
  if (loss_rows != nullptr && lane == 0) {
    const float zl = (lab >= 0 && lab < C) ? z[lab] : 0.f;
    loss_rows[r] = logf(se) + mx - zl;
  }
}

template <typename TD> __device__ __forceinline__ float get(const TD* p);
template <> __device__ __forceinline__ float get<float>(const float* p) { return *p; }
template <> __device__ __forceinline__ float get<__bf16>(const __bf16* p) {
  return static_cast<float>(*p);
}

// db[k][n] = sum_b dz[k][b][n].  A workgroup owns 64 adjacent columns of one replica; its four
// wavefronts take every fourth row (lane = column, so a row is one coalesced read), each lane
// keeps four partial sums, and the partials are combined in a fixed order through LDS.
template <typename TD>
__global__ __launch_bounds__(kThreads) void bias_grad_kernel(const TD* __restrict__ dz, long long ld,
                                                            float* __restrict__ db,
                                                            long long strideDb, int B, int N,
                                                            double* __restrict__ sumsq,
                                                            long long strideSumsq) {
  __shared__ float part[kWaves][64];
  const int k = blockIdx.y;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int n = blockIdx.x * 64 + lane;
  float s0 = 0.f, s1 = 0.f, s2 = 0.f, s3 = 0.f;
  if (n < N) {
    constexpr bool blocked = sizeof(TD) == 2;
    const int cb = b32s_blocks(N);
    const TD* base = blocked ? dz + (long long)k * ld : dz + (long long)k * B * ld + n;
    auto at = [&](int b) {
      return get<TD>(blocked ? base + b32s_offset(b, n, cb) : base + (long long)b * ld);
    };
    int b = wave;
    for (; b + 3 * kWaves < B; b += 4 * kWaves) {
      s0 += at(b);
      s1 += at(b + kWaves);
      s2 += at(b + 2 * kWaves);
      s3 += at(b + 3 * kWaves);
    }
    for (; b < B; b += kWaves) s0 += at(b);
  }
  part[wave][lane] = (s0 + s1) + (s2 + s3);
  __syncthreads();
  if (wave == 0) {
    float r = 0.f;
    if (n < N) {
      r = (part[0][lane] + part[1][lane]) + (part[2][lane] + part[3][lane]);
      db[(long long)k * strideDb + n] = r;
    }
    if (sumsq != nullptr) {        // sum of the squares of this workgroup's 64 results
      double q = (double)r * (double)r;
#pragma unroll
      for (int off = 32; off > 0; off >>= 1) q += __shfl_xor(q, off, 64);
      if (lane == 0) sumsq[(long long)k * strideSumsq + blockIdx.x] = q;
    }
  }
}

}  // namespace

void launch_softmax_ce(const float* logits, int ld, const int32_t* labels, void* dz, int64_t ld_dz,
                       int dz_bf16, float* loss_rows, int K, int B, int C, hipStream_t s) {
  const int rows = K * B;
  const unsigned grid = (rows + kWaves - 1) / kWaves;
  if (dz_bf16)
    softmax_ce_kernel<__bf16><<<grid, kThreads, 0, s>>>(logits, ld, labels, (__bf16*)dz, ld_dz,
                                                        loss_rows, rows, B, C);
  else
    softmax_ce_kernel<float><<<grid, kThreads, 0, s>>>(logits, ld, labels, (float*)dz, ld_dz,
                                                       loss_rows, rows, B, C);
}

int launch_bias_grad(const void* dz, int64_t ld, int dz_bf16, float* db, int64_t strideDb, int K,
                     int B, int N, double* sumsq, int64_t sumsq_stride, hipStream_t s) {
  dim3 grid((N + 63) / 64, K);
  if (dz_bf16)
    bias_grad_kernel<__bf16><<<grid, kThreads, 0, s>>>((const __bf16*)dz, ld, db, strideDb, B, N,
                                                       sumsq, sumsq_stride);
  else
    bias_grad_kernel<float><<<grid, kThreads, 0, s>>>((const float*)dz, ld, db, strideDb, B, N,
                                                      sumsq, sumsq_stride);
  return (int)grid.x;
}

}  // namespace lsam
