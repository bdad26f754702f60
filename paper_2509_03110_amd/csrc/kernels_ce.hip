// Fused softmax cross-entropy forward + backward (one wavefront per sample row, wavefront
// shuffle reductions) and the bias gradient (column sums of dZ).
#include <atomic>

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

// The same for dz in the blocked bf16 layout, read the way it is stored: a workgroup owns two
// adjacent column blocks (64 columns) of one replica, and per block row its 256 threads take the
// 4 KiB the two blocks occupy as one 16-byte unit each -- a thread keeps its position inside the
// block, so its 8 elements are the same 8 columns of the same row in every block row.  The 32
// threads that share 8 columns are then combined in row order through LDS.
__global__ __launch_bounds__(kThreads) void bias_grad_blocked_kernel(
    const __bf16* __restrict__ dz, long long stride, float* __restrict__ db, long long strideDb, int B,
    int N, double* __restrict__ sumsq, long long strideSumsq) {
  typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
  __shared__ float part[kThreads][9];            // pitch 9: the combining reads hit distinct banks
  const int k = blockIdx.y, t = threadIdx.x;
  const int cb = b32s_blocks(N), rbs = b32s_blocks(B);
  const int blk = blockIdx.x * 2 + (t >> 7);     // this thread's column block
  const int row = (t & 127) >> 2;                // its row inside a block
  float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  if (blk < cb) {
    const __bf16* p = dz + (long long)k * stride + (long long)blk * 1024 + (t & 127) * 8;
    const long long step = (long long)cb * 1024;
    auto add = [&](const u32x4& u) {
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        acc[2 * e] += __builtin_bit_cast(float, u[e] << 16);
        acc[2 * e + 1] += __builtin_bit_cast(float, u[e] & 0xFFFF0000u);
      }
    };
    int rb = 0;
    for (; rb + 3 < rbs && (rb + 3) * 32 + row < B; rb += 4) {
      const u32x4 u0 = *reinterpret_cast<const u32x4*>(p + rb * step);
      const u32x4 u1 = *reinterpret_cast<const u32x4*>(p + (rb + 1) * step);
      const u32x4 u2 = *reinterpret_cast<const u32x4*>(p + (rb + 2) * step);
      const u32x4 u3 = *reinterpret_cast<const u32x4*>(p + (rb + 3) * step);
      add(u0); add(u1); add(u2); add(u3);
    }
    for (; rb < rbs && rb * 32 + row < B; ++rb) add(*reinterpret_cast<const u32x4*>(p + rb * step));
  }
#pragma unroll
  for (int e = 0; e < 8; ++e) part[t][e] = acc[e];
  __syncthreads();
  if (t < 64) {
    // column c of this workgroup: block c / 32, unit q = (c % 32) / 8, element c % 8; in row r the
    // unit sits at position q ^ ((r / 4) % 4)
    const int n = blockIdx.x * 64 + t;
    const int q = (t & 31) >> 3, e = t & 7, base = (t >> 5) * 128;
    float r = 0.f;
    if (n < N) {
      for (int rr = 0; rr < 32; ++rr) r += part[base + rr * 4 + (q ^ ((rr >> 2) & 3))][e];
      db[(long long)k * strideDb + n] = r;
    }
    if (sumsq != nullptr) {        // sum of the squares of this workgroup's 64 results
      double sq = (double)r * (double)r;
#pragma unroll
      for (int off = 32; off > 0; off >>= 1) sq += __shfl_xor(sq, off, 64);
      if (t == 0) sumsq[(long long)k * strideSumsq + blockIdx.x] = sq;
    }
  }
}

// ---- narrow classifier head (fp32, at most 16 classes, at most 1024 inputs) ---------------------
// With C <= 16 outputs the last layer is three matrix products far too thin for MFMA tiles
// (forward [B x in] x [in x C], dX [B x C] x [C x in], dW [C x B] x [B x in]); as GEMMs each is
// a launch of its own (plus split-K reduce, softmax and bias gradient) that lasts 5-10 us
// whatever it computes.  Two kernels replace them.  Both are chains of memory latency, not of
// arithmetic, so each fetches everything it needs in one round of loads into LDS.
constexpr int kHeadMaxC = 16;
constexpr int kHeadMaxIn = 1024;     // padded input width that fits LDS beside the rows
constexpr int kHeadMaxB = 512;
constexpr int kHeadRows = 4;         // sample rows per workgroup, one per wavefront
typedef float hf4 __attribute__((ext_vector_type(4)));

// Forward, loss, dZ and masked dX of kHeadRows rows of one replica.  LDS: the C weight rows
// (pitch ld) then the sample rows (pitch ld); ld = input width rounded up to 8 = the pitch of
// both in memory, columns in..ld-1 hold zeros.
__global__ __launch_bounds__(kThreads) void head_forward_backward_kernel(
    const float* __restrict__ A, const float* __restrict__ W, const float* __restrict__ bias,
    long long strideW, const int32_t* __restrict__ labels, float* __restrict__ dz, int ld_dz,
    float* __restrict__ loss_rows, float* __restrict__ dA, int B, int C, int in, int ld) {
  extern __shared__ __attribute__((aligned(16))) float head_lds[];
  __shared__ float reds[kWaves][kHeadMaxC * 64];
  __shared__ float tot[kWaves][kHeadMaxC];
  float* Ws = head_lds;
  float* As = head_lds + C * ld;
  const int k = blockIdx.y;
  const int row0 = blockIdx.x * kHeadRows;
  const int nrows = B - row0 < kHeadRows ? B - row0 : kHeadRows;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const float* w = W + (long long)k * strideW;
  const float* a = A + ((long long)k * B + row0) * ld;
  for (int i = tid; i < C * ld / 4; i += kThreads)
    reinterpret_cast<hf4*>(Ws)[i] = reinterpret_cast<const hf4*>(w)[i];
  for (int i = tid; i < nrows * ld / 4; i += kThreads)
    reinterpret_cast<hf4*>(As)[i] = reinterpret_cast<const hf4*>(a)[i];
  __syncthreads();
  for (int rr = wave; rr < nrows; rr += kWaves) {
    const long long r = (long long)k * B + row0 + rr;
    const float* ar = As + rr * ld;
    float acc[kHeadMaxC];
#pragma unroll
    for (int c = 0; c < kHeadMaxC; ++c) acc[c] = 0.f;
    for (int j = lane * 4; j < ld; j += 256) {
      const hf4 av = *reinterpret_cast<const hf4*>(ar + j);
#pragma unroll
      for (int c = 0; c < kHeadMaxC; ++c)
        if (c < C) {
          const hf4 wv = *reinterpret_cast<const hf4*>(Ws + c * ld + j);
          acc[c] += (av[0] * wv[0] + av[1] * wv[1]) + (av[2] * wv[2] + av[3] * wv[3]);
        }
    }
    // Sum the 64 lanes' partial dot products: through the wavefront's LDS strip, lane l adding
    // 16 of the 64 partials of class l / 4, then two neighbour exchanges; every lane then reads
    // the C totals back.  (Sixty dependent cross-lane shuffles took longer than the products.)
    float* red = reds[wave];
#pragma unroll
    for (int c = 0; c < kHeadMaxC; ++c) red[c * 64 + lane] = acc[c];
    {
      const float* src = red + (lane >> 2) * 64 + (lane & 3) * 16;
      float t = 0.f;
#pragma unroll
      for (int q = 0; q < 16; ++q) t += src[q];
      t += __shfl_xor(t, 1, 64);
      t += __shfl_xor(t, 2, 64);
      tot[wave][lane >> 2] = t;
    }
    float d[kHeadMaxC];
    float mx = -INFINITY;
#pragma unroll
    for (int c = 0; c < kHeadMaxC; ++c) {
      d[c] = c < C ? tot[wave][c] + bias[(long long)k * strideW + c] : -INFINITY;   // logits
      mx = fmaxf(mx, d[c]);
    }
    float se = 0.f;
#pragma unroll
    for (int c = 0; c < kHeadMaxC; ++c)
      if (c < C) se += __expf(d[c] - mx);
    const int lab = labels[r];
    const float inv = 1.f / se, invB = 1.f / (float)B;
    float zl = 0.f;
#pragma unroll
    for (int c = 0; c < kHeadMaxC; ++c) {
      float v = 0.f;
      if (c < C) {
        v = __expf(d[c] - mx) * inv;
        if (c == lab) { v -= 1.f; zl = d[c]; }
        v *= invB;
      }
      d[c] = v;                                                                          // dZ
    }
    if (lane < ld_dz) {            // ld_dz <= 16: one lane per column, padding columns zero
      float v = 0.f;
#pragma unroll
      for (int q = 0; q < kHeadMaxC; ++q)
        if (q == lane) v = d[q];
      dz[r * ld_dz + lane] = v;
    }
    if (loss_rows != nullptr && lane == 0) loss_rows[r] = logf(se) + mx - zl;
    // dA = dZ W, kept where the layer's input (a ReLU output) is positive
    if (dA != nullptr) {
      for (int j = lane * 4; j < ld; j += 256) {
        const hf4 av = *reinterpret_cast<const hf4*>(ar + j);
        hf4 o = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int c = 0; c < kHeadMaxC; ++c)
          if (c < C) o += d[c] * *reinterpret_cast<const hf4*>(Ws + c * ld + j);
#pragma unroll
        for (int e = 0; e < 4; ++e)
          if (!(j + e < in && av[e] > 0.f)) o[e] = 0.f;
        *reinterpret_cast<hf4*>(dA + r * ld + j) = o;
      }
    }
  }
}

// dW[k][c][j] = sum_b dz[k][b][c] A[k][b][j] for 16 columns j of one replica, and (first
// workgroup of a replica) db[c] = sum_b dz[b][c].  Thread = (column, one of 16 row groups); the
// row groups are combined in a fixed order through LDS.  LDS (dynamic): dZ of the replica.
__global__ __launch_bounds__(kThreads) void head_weight_grad_kernel(
    const float* __restrict__ dz, int ld_dz, const float* __restrict__ A, int ldA,
    float* __restrict__ dW, int ldw, float* __restrict__ db, long long strideG, int B, int C,
    int in, double* __restrict__ sumsq, long long strideSumsq) {
  extern __shared__ __attribute__((aligned(16))) float head_lds[];
  __shared__ float part[16][kHeadMaxC][17];
  __shared__ double ssq_part[kWaves];
  float* dzs = head_lds;
  const int k = blockIdx.y;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int col = tid & 15, rg = tid >> 4;
  const float* dzk = dz + (long long)k * B * ld_dz;
  for (int i = tid; i < B * ld_dz / 4; i += kThreads)
    reinterpret_cast<hf4*>(dzs)[i] = reinterpret_cast<const hf4*>(dzk)[i];
  const int j = blockIdx.x * 16 + col;
  const float* ak = A + (long long)k * B * ldA + j;
  float acc[kHeadMaxC];
#pragma unroll
  for (int c = 0; c < kHeadMaxC; ++c) acc[c] = 0.f;
  __syncthreads();
  if (j < in) {
#pragma unroll 8
    for (int b = rg; b < B; b += 16) {
      const float av = ak[(long long)b * ldA];
#pragma unroll
      for (int c = 0; c < kHeadMaxC; ++c)
        if (c < C) acc[c] += dzs[b * ld_dz + c] * av;
    }
  }
#pragma unroll
  for (int c = 0; c < kHeadMaxC; ++c) part[rg][c][col] = acc[c];
  __syncthreads();
  float ssq = 0.f;
  {
    const int c = tid >> 4;                 // thread = (class, column)
    float v = 0.f;
#pragma unroll
    for (int q = 0; q < 16; ++q) v += part[q][c][col];
    if (c < C && j < in) {
      dW[(long long)k * strideG + (long long)c * ldw + j] = v;
      ssq += v * v;
    }
  }
  if (blockIdx.x == 0 && tid < C) {
    float s0 = 0.f, s1 = 0.f;
    int b = 0;
    for (; b + 1 < B; b += 2) { s0 += dzs[b * ld_dz + tid]; s1 += dzs[(b + 1) * ld_dz + tid]; }
    if (b < B) s0 += dzs[b * ld_dz + tid];
    const float sb = s0 + s1;
    db[(long long)k * strideG + tid] = sb;
    ssq += sb * sb;
  }
  if (sumsq != nullptr) {
    double q = (double)ssq;
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) q += __shfl_xor(q, off, 64);
    if (lane == 0) ssq_part[wave] = q;
    __syncthreads();
    if (tid == 0)
      sumsq[(long long)k * strideSumsq + blockIdx.x] =
          (ssq_part[0] + ssq_part[1]) + (ssq_part[2] + ssq_part[3]);
  }
}

}  // namespace

bool head_fits(int B, int C, int in) {
  return C <= kHeadMaxC && (in + 7) / 8 * 8 <= kHeadMaxIn && B <= kHeadMaxB;
}
int head_sumsq_slots(int in) { return (in + 15) / 16; }

int launch_head_forward_backward(const float* A, const float* W, const float* bias, int64_t strideW,
                                 const int32_t* labels, float* dz, int ld_dz, float* loss_rows,
                                 float* dA, int K, int B, int C, int in, hipStream_t s) {
  const int ld = (in + 7) / 8 * 8;
  const size_t lds = (size_t)(C + kHeadRows) * ld * 4;
  // the largest dynamic LDS size asked for so far (host threads may race here: the attribute
  // call is idempotent, the counter only saves repeating it)
  static std::atomic<size_t> granted{0};
  if (lds > granted.load(std::memory_order_relaxed)) {
    if (hipFuncSetAttribute(reinterpret_cast<const void*>(head_forward_backward_kernel),
                            hipFuncAttributeMaxDynamicSharedMemorySize,
                            (int)((size_t)(kHeadMaxC + kHeadRows) * kHeadMaxIn * 4)) != hipSuccess)
      return -1;
    granted.store((size_t)(kHeadMaxC + kHeadRows) * kHeadMaxIn * 4, std::memory_order_relaxed);
  }
  dim3 grid((B + kHeadRows - 1) / kHeadRows, K);
  head_forward_backward_kernel<<<grid, kThreads, lds, s>>>(A, W, bias, strideW, labels, dz, ld_dz,
                                                            loss_rows, dA, B, C, in, ld);
  return 0;
}

int launch_head_weight_grad(const float* dz, int ld_dz, const float* A, int ldA, float* dW, int ldw,
                            float* db, int64_t strideG, int K, int B, int C, int in, double* sumsq,
                            int64_t sumsq_stride, hipStream_t s) {
  dim3 grid(head_sumsq_slots(in), K);
  head_weight_grad_kernel<<<grid, kThreads, (size_t)B * ld_dz * 4, s>>>(
      dz, ld_dz, A, ldA, dW, ldw, db, strideG, B, C, in, sumsq, sumsq_stride);
  return (int)grid.x;
}

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
    bias_grad_blocked_kernel<<<grid, kThreads, 0, s>>>((const __bf16*)dz, ld, db, strideDb, B, N,
                                                       sumsq, sumsq_stride);
  else
    bias_grad_kernel<float><<<grid, kThreads, 0, s>>>((const float*)dz, ld, db, strideDb, B, N,
                                                      sumsq, sumsq_stride);
  return (int)grid.x;
}

}  // namespace lsam
