// Kernels around the 3x3 convolution layers of the convolutional model (Section "Experiments":
// the paper's workers train convolutional networks on 32x32x3 images).  A convolution with
// stride 1 and a zero rim of one pixel is run as a GEMM over the unfolded image
//   col[(b,i,j), (u,v,c)] = X[b, i+u-1, j+v-1, c]      (0 outside the image)
// so that the filter bank [out, 3, 3, C] is the GEMM's [out, 9 C] weight matrix and the
// tuned GEMM kernels serve forward, dW and dX unchanged.  This file holds what is left: the
// unfold and its adjoint (a gather: every input pixel sums its up to nine contributions in a
// fixed order), the 2x2 max-pool, and the pool's backward pass fused with the ReLU mask.
// All tensors are fp32, [K][B][H][W][C] with C contiguous; all four kernels are bandwidth
// bound and move 128-bit words, consecutive lanes on consecutive words.
#include "engine.h"

namespace lsam {
namespace {

constexpr int kThreads = 256;
typedef float f32x4 __attribute__((ext_vector_type(4)));

struct ImgShape {
  int H, W, C;     // one image
  int ld;          // pitch of a col row (floats), multiple of 4, >= 9 C
  long long rows;  // B H W
  long long total; // threads needed
};

// One thread per 16-byte word of col.  VEC: C % 4 == 0, a word then lies inside one tap.
template <bool VEC>
__global__ __launch_bounds__(kThreads) void unfold3x3_kernel(const float* __restrict__ X,
                                                             float* __restrict__ col, ImgShape sh,
                                                             long long strideX, long long strideCol) {
  const long long idx = (long long)blockIdx.x * kThreads + threadIdx.x;
  if (idx >= sh.total) return;
  const int words = sh.ld / 4;
  const int q = (int)(idx % words);
  long long m = idx / words;
  const int k = (int)(m / sh.rows);
  m -= (long long)k * sh.rows;
  const int j = (int)(m % sh.W);
  const int i = (int)((m / sh.W) % sh.H);
  const long long b = m / ((long long)sh.W * sh.H);
  const float* img = X + (long long)k * strideX + b * ((long long)sh.H * sh.W * sh.C);
  f32x4 o = {0.f, 0.f, 0.f, 0.f};
  if constexpr (VEC) {
    const int e = 4 * q;
    if (e < 9 * sh.C) {
      const int tap = e / sh.C, c = e - tap * sh.C;
      const int ii = i + tap / 3 - 1, jj = j + tap % 3 - 1;
      if (ii >= 0 && ii < sh.H && jj >= 0 && jj < sh.W)
        o = *reinterpret_cast<const f32x4*>(img + ((long long)ii * sh.W + jj) * sh.C + c);
    }
  } else {
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      const int e = 4 * q + r;
      if (e < 9 * sh.C) {
        const int tap = e / sh.C, c = e - tap * sh.C;
        const int ii = i + tap / 3 - 1, jj = j + tap % 3 - 1;
        if (ii >= 0 && ii < sh.H && jj >= 0 && jj < sh.W)
          o[r] = img[((long long)ii * sh.W + jj) * sh.C + c];
      }
    }
  }
  *reinterpret_cast<f32x4*>(col + (long long)k * strideCol + m * sh.ld + 4 * q) = o;
}

// Adjoint of the unfold: dX[b,i,j,c] = sum_{u,v} dcol[(b, i-u+1, j-v+1), (u,v,c)], taps in
// (u, v) order; with a mask, zero where mask <= 0 (the ReLU output the image came from).
// One thread per 16-byte word of dX; C % 4 == 0.
__global__ __launch_bounds__(kThreads) void fold3x3_kernel(const float* __restrict__ dcol,
                                                           float* __restrict__ dX,
                                                           const float* __restrict__ mask, ImgShape sh,
                                                           long long strideCol, long long strideX) {
  const long long idx = (long long)blockIdx.x * kThreads + threadIdx.x;
  if (idx >= sh.total) return;
  const int words = sh.C / 4;
  const int c = (int)(idx % words) * 4;
  long long m = idx / words;
  const int k = (int)(m / sh.rows);
  m -= (long long)k * sh.rows;
  const int j = (int)(m % sh.W);
  const int i = (int)((m / sh.W) % sh.H);
  const float* src = dcol + (long long)k * strideCol;
  f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
  for (int tap = 0; tap < 9; ++tap) {
    const int ii = i - (tap / 3 - 1), jj = j - (tap % 3 - 1);
    if (ii >= 0 && ii < sh.H && jj >= 0 && jj < sh.W) {
      const long long mm = m + (long long)(ii - i) * sh.W + (jj - j);
      acc += *reinterpret_cast<const f32x4*>(src + mm * sh.ld + tap * sh.C + c);
    }
  }
  const long long at = (long long)k * strideX + m * sh.C + c;
  if (mask != nullptr) {
    const f32x4 keep = *reinterpret_cast<const f32x4*>(mask + at);
#pragma unroll
    for (int r = 0; r < 4; ++r)
      if (!(keep[r] > 0.f)) acc[r] = 0.f;
  }
  *reinterpret_cast<f32x4*>(dX + at) = acc;
}

struct PoolShape {
  int Ho, Wo, C;    // pooled image
  long long cells;  // K B Ho Wo C/4
};

// P[b,i,j,c] = max over the 2x2 window of A.  One thread per 16-byte word of P.
__global__ __launch_bounds__(kThreads) void maxpool2_kernel(const float* __restrict__ A,
                                                            float* __restrict__ P, PoolShape sh) {
  const long long idx = (long long)blockIdx.x * kThreads + threadIdx.x;
  if (idx >= sh.cells) return;
  const int words = sh.C / 4;
  const int c = (int)(idx % words) * 4;
  long long cell = idx / words;          // (k b, i, j) of the pooled image
  const int j = (int)(cell % sh.Wo);
  const int i = (int)((cell / sh.Wo) % sh.Ho);
  const long long kb = cell / ((long long)sh.Wo * sh.Ho);
  const int W = 2 * sh.Wo;
  const float* a = A + ((kb * 2 * sh.Ho + 2 * i) * W + 2 * j) * sh.C + c;
  f32x4 m = *reinterpret_cast<const f32x4*>(a);
  const f32x4 v1 = *reinterpret_cast<const f32x4*>(a + sh.C);
  const f32x4 v2 = *reinterpret_cast<const f32x4*>(a + (long long)W * sh.C);
  const f32x4 v3 = *reinterpret_cast<const f32x4*>(a + (long long)W * sh.C + sh.C);
#pragma unroll
  for (int r = 0; r < 4; ++r) {
    m[r] = v1[r] > m[r] ? v1[r] : m[r];
    m[r] = v2[r] > m[r] ? v2[r] : m[r];
    m[r] = v3[r] > m[r] ? v3[r] : m[r];
  }
  *reinterpret_cast<f32x4*>(P + cell * sh.C + c) = m;
}

// Backward of ReLU followed by the pool: dA[window] = dP where A is the window's first
// maximum (row-major window order) and positive, else 0.  A is the ReLU output.
__global__ __launch_bounds__(kThreads) void maxpool2_backward_kernel(const float* __restrict__ A,
                                                                     const float* __restrict__ dP,
                                                                     float* __restrict__ dA,
                                                                     PoolShape sh) {
  const long long idx = (long long)blockIdx.x * kThreads + threadIdx.x;
  if (idx >= sh.cells) return;
  const int words = sh.C / 4;
  const int c = (int)(idx % words) * 4;
  long long cell = idx / words;
  const int j = (int)(cell % sh.Wo);
  const int i = (int)((cell / sh.Wo) % sh.Ho);
  const long long kb = cell / ((long long)sh.Wo * sh.Ho);
  const int W = 2 * sh.Wo;
  const long long base = ((kb * 2 * sh.Ho + 2 * i) * W + 2 * j) * sh.C + c;
  const long long offs[4] = {0, sh.C, (long long)W * sh.C, (long long)W * sh.C + sh.C};
  f32x4 v[4], o[4];
#pragma unroll
  for (int t = 0; t < 4; ++t) v[t] = *reinterpret_cast<const f32x4*>(A + base + offs[t]);
  const f32x4 g = *reinterpret_cast<const f32x4*>(dP + cell * sh.C + c);
#pragma unroll
  for (int r = 0; r < 4; ++r) {
    int best = 0;
    float m = v[0][r];
#pragma unroll
    for (int t = 1; t < 4; ++t)
      if (v[t][r] > m) { m = v[t][r]; best = t; }
#pragma unroll
    for (int t = 0; t < 4; ++t) o[t][r] = (t == best && m > 0.f) ? g[r] : 0.f;
  }
#pragma unroll
  for (int t = 0; t < 4; ++t) *reinterpret_cast<f32x4*>(dA + base + offs[t]) = o[t];
}

// First stage of the column sums of a tall matrix [rows][N] (N % 4 == 0, N <= 1024): workgroup
// (chunk, k) adds kColsumRows rows (short chunks: the matrices are tall and few, and the
// launch needs thousands of workgroups to use the memory system).  Thread = (column word, row group); the row groups are
// combined through LDS in a fixed order.
constexpr int kColsumRows = 256;
__global__ __launch_bounds__(kThreads) void colsum_partial_kernel(const float* __restrict__ A,
                                                                  float* __restrict__ partial,
                                                                  long long rows, int N, int chunks) {
  __shared__ f32x4 part[kThreads];
  const int words = N / 4;
  const int groups = kThreads / words;
  const int w = threadIdx.x % words, grp = threadIdx.x / words;
  const int k = blockIdx.y;
  const long long r0 = (long long)blockIdx.x * kColsumRows;
  const long long r1 = r0 + kColsumRows < rows ? r0 + kColsumRows : rows;
  f32x4 acc = {0.f, 0.f, 0.f, 0.f};
  if (grp < groups) {
    const float* base = A + ((long long)k * rows) * N + 4 * w;
    for (long long r = r0 + grp; r < r1; r += groups) acc += *reinterpret_cast<const f32x4*>(base + r * N);
  }
  part[threadIdx.x] = acc;
  __syncthreads();
  if (threadIdx.x < words) {
    f32x4 tot = part[threadIdx.x];
    for (int gq = 1; gq < groups; ++gq) tot += part[gq * words + threadIdx.x];
    *reinterpret_cast<f32x4*>(partial + ((long long)k * chunks + blockIdx.x) * N + 4 * threadIdx.x) = tot;
  }
}

// Wt[k][c][(u,v,o)] = W[k][o][(2-u, 2-v, c)]: the filter bank as the weight matrix of the
// convolution that maps the output gradient back to the input (taps mirrored, channels
// swapped).  One thread per element of Wt, o fastest.
__global__ __launch_bounds__(kThreads) void flip_filters_kernel(const float* __restrict__ W,
                                                                long long strideW, int ldw,
                                                                float* __restrict__ Wt, int Cout,
                                                                int Cin, long long total) {
  const long long idx = (long long)blockIdx.x * kThreads + threadIdx.x;
  if (idx >= total) return;
  const int o = (int)(idx % Cout);
  long long rest = idx / Cout;
  const int tap = (int)(rest % 9);
  rest /= 9;
  const int c = (int)(rest % Cin);
  const long long k = rest / Cin;
  Wt[idx] = W[k * strideW + (long long)o * ldw + (8 - tap) * Cin + c];
}

unsigned blocks_for(long long total) { return (unsigned)((total + kThreads - 1) / kThreads); }

}  // namespace

int launch_unfold3x3(const float* X, int64_t strideX, float* col, int64_t strideCol, int ld, int K,
                     int B, int H, int W, int C, hipStream_t s) {
  ImgShape sh{H, W, C, ld, (long long)B * H * W, 0};
  sh.total = (long long)K * sh.rows * (ld / 4);
  if (ld % 4 || ld < 9 * C || sh.total <= 0 || sh.total >= (1ll << 31) * kThreads) return -1;
  if (C % 4 == 0)
    unfold3x3_kernel<true><<<blocks_for(sh.total), kThreads, 0, s>>>(X, col, sh, strideX, strideCol);
  else
    unfold3x3_kernel<false><<<blocks_for(sh.total), kThreads, 0, s>>>(X, col, sh, strideX, strideCol);
  return 0;
}

int launch_fold3x3(const float* dcol, int64_t strideCol, int ld, float* dX, const float* mask,
                   int64_t strideX, int K, int B, int H, int W, int C, hipStream_t s) {
  ImgShape sh{H, W, C, ld, (long long)B * H * W, 0};
  sh.total = (long long)K * sh.rows * (C / 4);
  if (C % 4 || ld < 9 * C || sh.total <= 0 || sh.total >= (1ll << 31) * kThreads) return -1;
  fold3x3_kernel<<<blocks_for(sh.total), kThreads, 0, s>>>(dcol, dX, mask, sh, strideCol, strideX);
  return 0;
}

void launch_flip_filters(const float* W, int64_t strideW, int ldw, float* Wt, int K, int Cout, int Cin,
                         hipStream_t s) {
  const long long total = (long long)K * Cin * 9 * Cout;
  flip_filters_kernel<<<blocks_for(total), kThreads, 0, s>>>(W, strideW, ldw, Wt, Cout, Cin, total);
}

int colsum_chunks(int64_t rows) { return (int)((rows + kColsumRows - 1) / kColsumRows); }

int launch_colsum_partials(const float* A, int64_t rows, int N, int K, float* partial, hipStream_t s) {
  if (N % 4 || N < 4 || N > 4 * kThreads || rows < 1) return -1;
  const int chunks = colsum_chunks(rows);
  colsum_partial_kernel<<<dim3((unsigned)chunks, (unsigned)K), kThreads, 0, s>>>(A, partial, rows, N,
                                                                                 chunks);
  return chunks;
}

int launch_maxpool2(const float* A, float* P, int64_t images, int H, int W, int C, hipStream_t s) {
  PoolShape sh{H / 2, W / 2, C, images * (H / 2) * (W / 2) * (C / 4)};
  if (C % 4 || H % 2 || W % 2 || sh.cells <= 0 || sh.cells >= (1ll << 31) * kThreads) return -1;
  maxpool2_kernel<<<blocks_for(sh.cells), kThreads, 0, s>>>(A, P, sh);
  return 0;
}

int launch_maxpool2_backward(const float* A, const float* dP, float* dA, int64_t images, int H,
                             int W, int C, hipStream_t s) {
  PoolShape sh{H / 2, W / 2, C, images * (H / 2) * (W / 2) * (C / 4)};
  if (C % 4 || H % 2 || W % 2 || sh.cells <= 0 || sh.cells >= (1ll << 31) * kThreads) return -1;
  maxpool2_backward_kernel<<<blocks_for(sh.cells), kThreads, 0, s>>>(A, dP, dA, sh);
  return 0;
}

}  // namespace lsam
