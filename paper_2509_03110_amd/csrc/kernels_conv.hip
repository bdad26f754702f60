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
  int H, W, C;     // one output image of the convolution (H x W positions), C input channels
  int ld;          // pitch of a col row (floats), multiple of 4, >= 9 C
  long long rows;  // B H W
  long long total; // threads needed
  int st;          // stride: the input image is [st H][st W][C]
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
  const int Hin = sh.st * sh.H, Win = sh.st * sh.W;
  const float* img = X + (long long)k * strideX + b * ((long long)Hin * Win * sh.C);
  f32x4 o = {0.f, 0.f, 0.f, 0.f};
  if constexpr (VEC) {
    const int e = 4 * q;
    if (e < 9 * sh.C) {
      const int tap = e / sh.C, c = e - tap * sh.C;
      const int ii = sh.st * i + tap / 3 - 1, jj = sh.st * j + tap % 3 - 1;
      if (ii >= 0 && ii < Hin && jj >= 0 && jj < Win)
        o = *reinterpret_cast<const f32x4*>(img + ((long long)ii * Win + jj) * sh.C + c);
    }
  } else {
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      const int e = 4 * q + r;
      if (e < 9 * sh.C) {
        const int tap = e / sh.C, c = e - tap * sh.C;
        const int ii = sh.st * i + tap / 3 - 1, jj = sh.st * j + tap % 3 - 1;
        if (ii >= 0 && ii < Hin && jj >= 0 && jj < Win)
          o[r] = img[((long long)ii * Win + jj) * sh.C + c];
      }
    }
  }
  *reinterpret_cast<f32x4*>(col + (long long)k * strideCol + m * sh.ld + 4 * q) = o;
}

// Adjoint of the unfold: dX[b,y,x,c] = sum over the taps (u,v) and output positions (i,j) with
// st i + u - 1 = y, st j + v - 1 = x of dcol[(b,i,j), (u,v,c)], taps in (u, v) order; with a
// mask, zero where mask <= 0 (the ReLU output the image came from).
// One thread per 16-byte word of dX; C % 4 == 0.  sh.rows counts the pixels of dX here.
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
  const int Hin = sh.st * sh.H, Win = sh.st * sh.W;
  const int x = (int)(m % Win);
  const int y = (int)((m / Win) % Hin);
  const long long b = m / ((long long)Win * Hin);
  const float* src = dcol + (long long)k * strideCol;
  f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
  for (int tap = 0; tap < 9; ++tap) {
    const int yy = y - (tap / 3 - 1), xx = x - (tap % 3 - 1);     // st i and st j
    if (yy >= 0 && xx >= 0 && yy % sh.st == 0 && xx % sh.st == 0) {
      const int ii = yy / sh.st, jj = xx / sh.st;
      if (ii < sh.H && jj < sh.W) {
        const long long mm = (b * sh.H + ii) * sh.W + jj;
        acc += *reinterpret_cast<const f32x4*>(src + mm * sh.ld + tap * sh.C + c);
      }
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

// Column reductions over the rows of tall matrices [K][rows][C] (C % 4 == 0) are done in two
// fixed-order stages.  First stage: workgroup (chunk, k, column block) covers `chunk_rows` rows
// of 64 columns; thread = (column word w of 16, row group of 16), each group strides over the
// chunk's rows, the groups are added in group order through LDS.  chunk_rows shrinks from 256
// towards 32 until the launch has about a thousand workgroups (short matrices would otherwise
// leave most of the chip idle behind a few long serial sums).
struct ChunkPlan {
  int chunk_rows, chunks, col_blocks;
};
ChunkPlan chunk_plan(long long rows, int C, int K) {
  ChunkPlan p;
  p.col_blocks = (C + 63) / 64;
  p.chunk_rows = 256;
  while (p.chunk_rows > 32 &&
         ((rows + p.chunk_rows - 1) / p.chunk_rows) * p.col_blocks * K < 1024)
    p.chunk_rows /= 2;
  p.chunks = (int)((rows + p.chunk_rows - 1) / p.chunk_rows);
  return p;
}
struct ChunkThread {
  int cw;          // column word (4 columns) of this thread
  int grp;         // row group 0..15
  bool live;       // the column word exists
  long long r0, r1;
};
__device__ __forceinline__ ChunkThread chunk_thread(long long rows, int C, int chunk_rows) {
  ChunkThread t;
  t.cw = blockIdx.z * 16 + (threadIdx.x & 15);
  t.grp = threadIdx.x >> 4;
  t.live = t.cw < C / 4;
  t.r0 = (long long)blockIdx.x * chunk_rows;
  t.r1 = t.r0 + chunk_rows < rows ? t.r0 + chunk_rows : rows;
  return t;
}
// Adds `v` over the 16 row groups in group order; the result is valid for grp == 0.
__device__ __forceinline__ f32x4 combine_groups(f32x4 v, const ChunkThread& t, f32x4* buf) {
  __syncthreads();
  buf[threadIdx.x] = v;
  __syncthreads();
  f32x4 tot = v;
  if (t.grp == 0)
    for (int gq = 1; gq < 16; ++gq) tot += buf[gq * 16 + (threadIdx.x & 15)];
  return tot;
}

// partial[k][chunk][c] = sum of the chunk's rows of A.
__global__ __launch_bounds__(kThreads) void colsum_partial_kernel(const float* __restrict__ A,
                                                                  float* __restrict__ partial,
                                                                  long long rows, int N, int chunks,
                                                                  int chunk_rows) {
  __shared__ f32x4 buf[kThreads];
  const ChunkThread t = chunk_thread(rows, N, chunk_rows);
  const int k = blockIdx.y;
  f32x4 acc = {0.f, 0.f, 0.f, 0.f};
  if (t.live) {
    const float* base = A + ((long long)k * rows) * N + 4 * t.cw;
    for (long long r = t.r0 + t.grp; r < t.r1; r += 16) acc += *reinterpret_cast<const f32x4*>(base + r * N);
  }
  const f32x4 tot = combine_groups(acc, t, buf);
  if (t.live && t.grp == 0)
    *reinterpret_cast<f32x4*>(partial + ((long long)k * chunks + blockIdx.x) * N + 4 * t.cw) = tot;
}

// Wt[k][c][(u,v,o)] = W[k][o][(2-u, 2-v, c)]: the filter bank as the weight matrix of the
// convolution that maps the output gradient back to the input (taps mirrored, channels
// swapped).  A 32 x 32 (o, c) tile of one tap per workgroup, transposed through LDS so that both
// the reads (c contiguous) and the writes (o contiguous) are whole 128-byte rows.  32 | Cout.
__global__ __launch_bounds__(kThreads) void flip_filters_kernel(const float* __restrict__ W,
                                                                long long strideW, int ldw,
                                                                float* __restrict__ Wt, int Cout,
                                                                int Cin, int cblocks) {
  __shared__ float tile[32][33];
  const int ob = (blockIdx.x / cblocks) * 32, cb = (blockIdx.x % cblocks) * 32;
  const int tap = blockIdx.y;
  const long long k = blockIdx.z;
  const int x = threadIdx.x & 31, y = threadIdx.x >> 5;
  const float* src = W + k * strideW + (long long)(8 - tap) * Cin;
#pragma unroll
  for (int r = 0; r < 32; r += 8)
    tile[y + r][x] = cb + x < Cin ? src[(long long)(ob + y + r) * ldw + cb + x] : 0.f;
  __syncthreads();
  float* dst = Wt + k * (long long)Cin * 9 * Cout + (long long)tap * Cout + ob + x;
#pragma unroll
  for (int r = 0; r < 32; r += 8)
    if (cb + y + r < Cin) dst[(long long)(cb + y + r) * 9 * Cout] = tile[x][y + r];
}

// ---- first convolution layer (1..3 input channels) -------------------------------------------------
// With C <= 3 the contraction is 9 C <= 27 long: too short to be worth staging through LDS, and
// a 16-byte unit of the unfolded image would straddle taps.  These two kernels feed the MFMA
// units (v_mfma_f32_32x32x2_f32) straight from global memory instead: every lane gathers the
// image values of its pixel (the image of one replica is a few MB and stays in cache), the
// filters sit in registers.  Lane (l32, h) supplies element (index l32, k = h) of each operand;
// accumulator element e of a lane belongs to (second operand's index l32, first operand's
// index (e/4)*8 + h*4 + e%4).
typedef float f32x16 __attribute__((ext_vector_type(16)));

struct FirstConv {
  int H, W, Cout;
  float invW, invH;
  long long rows;          // B H W pixels per replica
  long long strideParams;  // floats between replicas' parameter (or gradient) vectors
  int ldw;                 // row pitch of the filter bank [Cout][9 C (+ padding)]
};

__device__ __forceinline__ void pixel_rc(int p, const FirstConv& f, int& i, int& j) {
  int q = (int)((float)p * f.invW);
  int r = p - q * f.W;
  if (r < 0) { r += f.W; --q; } else if (r >= f.W) { r -= f.W; ++q; }
  j = r;
  const int q2 = (int)((float)q * f.invH);
  int r2 = q - q2 * f.H;
  if (r2 < 0) r2 += f.H; else if (r2 >= f.H) r2 -= f.H;
  i = r2;
}

// bfloat16 value nearest to v (ties to even), as a float: products of two such values are exact
// in fp32, so fp32 MFMAs on rounded operands give what the bf16 matrix instructions give.
__device__ __forceinline__ float to_bf16(float v) { return static_cast<float>(static_cast<__bf16>(v)); }

// Value t of the unfolded image of pixel p at (i, j): X[p shifted by tap t / C][t % C].
template <int C>
__device__ __forceinline__ float unfolded(const float* __restrict__ img, int p, int i, int j, int t,
                                          const FirstConv& f) {
  const int tap = t / C, c = t - tap * C;
  const int du = tap / 3 - 1, dv = tap % 3 - 1;
  const bool ok = tap < 9 && (unsigned)(i + du) < (unsigned)f.H && (unsigned)(j + dv) < (unsigned)f.W;
  return ok ? img[(long long)(p + du * f.W + dv) * C + c] : 0.f;
}

// out[k][p][o] = relu(b[o] + sum_t unfolded(p, t) W[o][t]).  One wavefront per 32 pixels.
template <int C>
__global__ __launch_bounds__(kThreads) void first_conv_forward_kernel(const float* __restrict__ X,
                                                                      const float* __restrict__ params,
                                                                      long long w_off, long long b_off,
                                                                      float* __restrict__ out,
                                                                      FirstConv f, int relu, int round) {
  constexpr int KS = (9 * C + 1) / 2;          // MFMA steps of depth 2
  constexpr int WP = 33;                       // LDS pitch of a filter: lanes o, o+1 on different banks
  extern __shared__ float wl[];                // [Cout][WP]: the filters, zero for t >= 9 C
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int l32 = lane & 31, h = lane >> 5;
  const int k = blockIdx.y;
  {
    // rows of 32 floats (lanes along t: whole 128-byte lines of the filter bank)
    const float* Wg = params + (long long)k * f.strideParams + w_off;
    for (int e = threadIdx.x; e < f.Cout * 32; e += kThreads) {
      const int o = e >> 5, t = e & 31;
      const float wv = t < 9 * C ? Wg[(long long)o * f.ldw + t] : 0.f;
      wl[o * WP + t] = round ? to_bf16(wv) : wv;
    }
  }
  __syncthreads();
  const int p = (blockIdx.x * 4 + wave) * 32 + l32;
  const bool live = p < f.rows;
  const float* img = X + (long long)k * f.rows * C;
  const float* bias = params + (long long)k * f.strideParams + b_off;
  int i = 0, j = 0;
  if (live) pixel_rc(p, f, i, j);
  float x[KS];
#pragma unroll
  for (int s = 0; s < KS; ++s) {
    x[s] = live ? unfolded<C>(img, p, i, j, 2 * s + h, f) : 0.f;
    if (round) x[s] = to_bf16(x[s]);
  }
  // acc[e] of lane (l32, h): output channel ob + l32 of pixel tile*32 + (e/4)*8 + h*4 + e%4, so
  // that a store instruction writes two whole 128-byte rows
  const int tile0 = (blockIdx.x * 4 + wave) * 32;
  for (int ob = 0; ob < f.Cout; ob += 32) {
    f32x16 acc;
#pragma unroll
    for (int e = 0; e < 16; ++e) acc[e] = 0.f;
#pragma unroll
    for (int s = 0; s < KS; ++s) {
      const float w = wl[(ob + l32) * WP + 2 * s + h];
      acc = __builtin_amdgcn_mfma_f32_32x32x2f32(x[s], w, acc, 0, 0, 0);
    }
    const float bv = bias[ob + l32];
    float* dst = out + ((long long)k * f.rows + tile0) * f.Cout + ob + l32;
#pragma unroll
    for (int e = 0; e < 16; ++e) {
      const int pp = (e / 4) * 8 + h * 4 + e % 4;
      const float z = acc[e] + bv;
      if (tile0 + pp < f.rows) dst[(long long)pp * f.Cout] = (relu && !(z > 0.f)) ? 0.f : z;
    }
  }
}

// Weight and bias gradient, first stage: workgroup (chunk, k) covers kFirstChunk pixels, 128 per
// wavefront; partial[k][chunk][o][t] = sum over its pixels of dout[p][o] unfolded(p, t), with
// t = 9 C standing for the constant 1 (that column is the bias gradient).  The four
// wavefronts' sums are added in wave order through LDS.
constexpr int kFirstChunk = 512;
template <int C>
__global__ __launch_bounds__(kThreads) void first_conv_wgrad_kernel(const float* __restrict__ X,
                                                                    const float* __restrict__ dout,
                                                                    float* __restrict__ partial,
                                                                    int chunks, FirstConv f, int round) {
  __shared__ float red[3][32 * 32];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int l32 = lane & 31, h = lane >> 5;
  const int k = blockIdx.y;
  const float* img = X + (long long)k * f.rows * C;
  const float* dz = dout + (long long)k * f.rows * f.Cout;
  const int p0 = blockIdx.x * kFirstChunk + wave * (kFirstChunk / 4);
  // this lane's column of the unfolded image: fixed tap and channel
  const int t = l32;
  const int tap = t / C, c = t - tap * C;
  const int du = tap / 3 - 1, dv = tap % 3 - 1;
  const int shift = (du * f.W + dv) * C + c;
  for (int ob = 0; ob < f.Cout; ob += 32) {
    f32x16 acc;
#pragma unroll
    for (int e = 0; e < 16; ++e) acc[e] = 0.f;
    // loads are issued unconditionally (from a clamped pixel) and zeroed afterwards, so that the
    // unrolled loop can have many of them in flight
    const int last = (int)f.rows - 1;
#pragma unroll 8
    for (int s = 0; s < kFirstChunk / 8; ++s) {
      const int p = p0 + 2 * s + h;
      const int pc = p < last ? p : last;
      int i, j;
      pixel_rc(pc, f, i, j);
      const bool in_img = t < 9 * C && (unsigned)(i + du) < (unsigned)f.H && (unsigned)(j + dv) < (unsigned)f.W;
      float a = dz[(long long)pc * f.Cout + ob + l32];
      float b = img[in_img ? (long long)pc * C + shift : 0];
      b = in_img ? b : (t == 9 * C ? 1.f : 0.f);
      if (p > last) { a = 0.f; b = 0.f; }
      if (round) { a = to_bf16(a); b = to_bf16(b); }
      acc = __builtin_amdgcn_mfma_f32_32x32x2f32(b, a, acc, 0, 0, 0);
    }
    // acc[e]: o = ob + l32, t = (e/4)*8 + h*4 + e%4
    if (wave > 0) {
#pragma unroll
      for (int e = 0; e < 16; ++e) red[wave - 1][l32 * 32 + (e / 4) * 8 + h * 4 + e % 4] = acc[e];
    }
    __syncthreads();
    if (wave == 0) {
      float* dst = partial + (((long long)k * chunks + blockIdx.x) * f.Cout + ob + l32) * 32;
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const int tt = q * 8 + h * 4;
        f32x4 v;
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          const int at = l32 * 32 + tt + r;
          v[r] = ((acc[q * 4 + r] + red[0][at]) + red[1][at]) + red[2][at];
        }
        *reinterpret_cast<f32x4*>(dst + tt) = v;
      }
    }
    __syncthreads();
  }
}

// Second stage: dW[k][o][t] (t < 9 C) and db[k][o] (t = 9 C) = sum over the chunks.  Workgroup
// (block, k) finishes 64 elements with 16 chains of loads each (chain q adds chunks q, q+16,
// ...), combined pairwise in a fixed tree through LDS; it also writes the sum of the squares of
// what it stored to its own slot.
constexpr int kFinishChains = 16;
__global__ __launch_bounds__(1024) void first_conv_wgrad_finish_kernel(const float* __restrict__ partial,
                                                                       int chunks, int C,
                                                                       float* __restrict__ grad,
                                                                       long long w_off, long long b_off,
                                                                       double* __restrict__ sumsq,
                                                                       long long strideSumsq,
                                                                       FirstConv f, int skip_bias) {
  __shared__ float part[kFinishChains][64];
  const int word = threadIdx.x & 63, q = threadIdx.x >> 6;
  const int k = blockIdx.y;
  const int total = f.Cout * 32;
  const int e = blockIdx.x * 64 + word;       // o * 32 + t; total is a multiple of 64
  float v = 0.f;
  for (int ch = q; ch < chunks; ch += kFinishChains) v += partial[((long long)k * chunks + ch) * total + e];
  part[q][word] = v;
  __syncthreads();
#pragma unroll
  for (int half = kFinishChains / 2; half > 0; half >>= 1) {
    if (q < half) part[q][word] += part[q + half][word];
    __syncthreads();
  }
  if (q == 0) {
    v = part[0][word];
    float* g = grad + (long long)k * f.strideParams;
    const int o = e >> 5, t = e & 31;
    double ssq = 0.0;
    if (t < 9 * C) { g[w_off + (long long)o * f.ldw + t] = v; ssq = (double)v * (double)v; }
    else if (t == 9 * C && !skip_bias) { g[b_off + o] = v; ssq = (double)v * (double)v; }
    if (sumsq != nullptr) {
#pragma unroll
      for (int off = 32; off > 0; off >>= 1) ssq += __shfl_xor(ssq, off, 64);
      if (word == 0) sumsq[(long long)k * strideSumsq + blockIdx.x] = ssq;
    }
  }
}

// ---- batch normalisation (training mode, per replica and channel over the B H W rows) -------------
// (Appendix "Batch Normalization": each worker uses the statistics of its own minibatch.)
// Z is [K][rows][C] (C % 4 == 0, C <= 1024).  Statistics in one pass over Z that does not lose
// digits when |mean| >> spread: every chunk of rows gets its own mean and its own sum of
// squared deviations from that mean (computed around the chunk's first row); the chunks are
// then combined in double, in a fixed order.
// (Chunks and thread layout: see colsum_partial_kernel.)
__global__ __launch_bounds__(kThreads) void bn_stats_partial_kernel(const float* __restrict__ Z,
                                                                    float* __restrict__ pmean,
                                                                    float* __restrict__ pm2,
                                                                    long long rows, int C, int chunks,
                                                                    int chunk_rows) {
  __shared__ f32x4 buf[kThreads];
  const ChunkThread t = chunk_thread(rows, C, chunk_rows);
  const int k = blockIdx.y;
  const float* base = Z + ((long long)k * rows) * C + 4 * t.cw;
  // One sweep: sums of (z - z0) and (z - z0)^2 with z0 the chunk's first row, a value of the
  // data's own size, so neither sum loses digits to a mean far from zero; then
  //   mean = z0 + s1 / n,   M2 = s2 - s1^2 / n.
  f32x4 s1 = {0.f, 0.f, 0.f, 0.f}, s2 = {0.f, 0.f, 0.f, 0.f}, z0 = {0.f, 0.f, 0.f, 0.f};
  if (t.live) {
    z0 = *reinterpret_cast<const f32x4*>(base + t.r0 * C);
    for (long long r = t.r0 + t.grp; r < t.r1; r += 16) {
      const f32x4 dlt = *reinterpret_cast<const f32x4*>(base + r * C) - z0;
      s1 += dlt;
      s2 += dlt * dlt;
    }
  }
  const f32x4 t1 = combine_groups(s1, t, buf);
  const f32x4 t2 = combine_groups(s2, t, buf);
  if (t.live && t.grp == 0) {
    const float inv_n = 1.f / (float)(t.r1 - t.r0);
    const long long at = ((long long)k * chunks + blockIdx.x) * C + 4 * t.cw;
    *reinterpret_cast<f32x4*>(pmean + at) = z0 + t1 * inv_n;
    f32x4 m2 = t2 - t1 * t1 * inv_n;
#pragma unroll
    for (int r = 0; r < 4; ++r) m2[r] = m2[r] > 0.f ? m2[r] : 0.f;
    *reinterpret_cast<f32x4*>(pm2 + at) = m2;
  }
}

// stats[k][0][c] = mean, stats[k][1][c] = 1 / sqrt(var + eps), var = M2 / rows (biased):
//   mean = sum_i n_i mean_i / rows,   M2 = sum_i [M2_i + n_i (mean_i - mean)^2]
// over the chunks i, in double.  Workgroup (block, k) serves 64 columns with 16 chains each
// (chain q takes chunks q, q + 16, ...); the chains are added in a fixed tree through LDS.
constexpr int kBnChains = 16;
__device__ __forceinline__ double chain_total(double v, double (*buf)[64], int q, int col) {
  __syncthreads();
  buf[q][col] = v;
  __syncthreads();
#pragma unroll
  for (int half = kBnChains / 2; half > 0; half >>= 1) {
    if (q < half) buf[q][col] += buf[q + half][col];
    __syncthreads();
  }
  return buf[0][col];
}
__global__ __launch_bounds__(64 * kBnChains) void bn_stats_finish_kernel(
    const float* __restrict__ pmean, const float* __restrict__ pm2, float* __restrict__ stats,
    long long rows, int C, int chunks, int chunk_rows, float eps) {
  __shared__ double buf[kBnChains][64];
  const int col = threadIdx.x & 63, q = threadIdx.x >> 6;
  const int c = blockIdx.x * 64 + col;
  const int k = blockIdx.y;
  const bool live = c < C;
  auto count = [&](int ch) {
    const long long left = rows - (long long)ch * chunk_rows;
    return (double)(left < chunk_rows ? left : chunk_rows);
  };
  double s1 = 0.0;
  if (live)
    for (int ch = q; ch < chunks; ch += kBnChains)
      s1 += count(ch) * (double)pmean[((long long)k * chunks + ch) * C + c];
  const double mean = chain_total(s1, buf, q, col) / (double)rows;
  double s2 = 0.0;
  if (live)
    for (int ch = q; ch < chunks; ch += kBnChains) {
      const long long at = ((long long)k * chunks + ch) * C + c;
      const double dlt = (double)pmean[at] - mean;
      s2 += (double)pm2[at] + count(ch) * dlt * dlt;
    }
  const double m2 = chain_total(s2, buf, q, col);
  if (live && q == 0) {
    stats[((long long)k * 2) * C + c] = (float)mean;
    stats[((long long)k * 2 + 1) * C + c] = (float)(1.0 / sqrt(m2 / (double)rows + (double)eps));
  }
}

// The shortcut of a residual block as the kernels read it: the block input [B][st H][st W][Cs]
// seen from an output pixel (i, j) and channel c is src[b][st i][st j][c] for c < Cs, 0 beyond.
// A projection shortcut instead: pz [K][rows][C] is the 1x1 convolution of the block input,
// normalised here with its own statistics pstats and gamma_p, beta_p (offsets into params).
struct Shortcut {
  const float* src;     // null: no parameter-free shortcut
  long long stride;     // floats from one replica's block input to the next
  int H, W, Cs, st;     // output image, channels of the block input, pixel step
  const float* pz;      // null: no projection
  const float* pstats;
  long long pgam_off, pbet_off;
};

// out = relu(gamma (Z - mean) inv_std + beta [+ shortcut]).  One thread per 16-byte word.
__global__ __launch_bounds__(kThreads) void bn_apply_kernel(const float* __restrict__ Z,
                                                            const float* __restrict__ stats,
                                                            const float* __restrict__ params,
                                                            long long strideParams, long long gam_off,
                                                            long long bet_off, float* __restrict__ out,
                                                            long long rows, int C, long long total,
                                                            Shortcut sc) {
  const long long idx = (long long)blockIdx.x * kThreads + threadIdx.x;
  if (idx >= total) return;
  const int words = C / 4;
  const int c = (int)(idx % words) * 4;
  const int k = (int)(idx / words / rows);
  const f32x4 mu = *reinterpret_cast<const f32x4*>(stats + ((long long)k * 2) * C + c);
  const f32x4 inv = *reinterpret_cast<const f32x4*>(stats + ((long long)k * 2 + 1) * C + c);
  const f32x4 ga = *reinterpret_cast<const f32x4*>(params + k * strideParams + gam_off + c);
  const f32x4 be = *reinterpret_cast<const f32x4*>(params + k * strideParams + bet_off + c);
  const f32x4 z = *reinterpret_cast<const f32x4*>(Z + idx * 4);
  f32x4 y = ga * ((z - mu) * inv) + be;
  if (sc.pz != nullptr) {
    const f32x4 pmu = *reinterpret_cast<const f32x4*>(sc.pstats + ((long long)k * 2) * C + c);
    const f32x4 pinv = *reinterpret_cast<const f32x4*>(sc.pstats + ((long long)k * 2 + 1) * C + c);
    const f32x4 pga = *reinterpret_cast<const f32x4*>(params + k * strideParams + sc.pgam_off + c);
    const f32x4 pbe = *reinterpret_cast<const f32x4*>(params + k * strideParams + sc.pbet_off + c);
    y += pga * ((*reinterpret_cast<const f32x4*>(sc.pz + idx * 4) - pmu) * pinv) + pbe;
  } else if (sc.src != nullptr && c < sc.Cs) {       // Cs % 4 == 0: a word lies inside or outside
    const long long m = idx / words - (long long)k * rows;       // (b, i, j) of this replica
    const int j = (int)(m % sc.W), i = (int)((m / sc.W) % sc.H);
    const long long b = m / ((long long)sc.W * sc.H);
    const long long at = ((b * (sc.st * sc.H) + sc.st * i) * (sc.st * sc.W) + sc.st * j) * sc.Cs + c;
    y += *reinterpret_cast<const f32x4*>(sc.src + k * sc.stride + at);
  }
#pragma unroll
  for (int r = 0; r < 4; ++r) y[r] = y[r] > 0.f ? y[r] : 0.f;
  *reinterpret_cast<f32x4*>(out + idx * 4) = y;
}

// The shortcut's share of the block input's gradient: dIn[b][st i][st j][c] += dY[b][i][j][c]
// for c < Cs (dY: gradient of the block output behind its ReLU), where the block input, itself
// a ReLU output `mask`, is positive (mask null: no such condition, the input came from a
// pool).  One thread per 16-byte word of the part of dY that has a counterpart.
__global__ __launch_bounds__(kThreads) void shortcut_backward_kernel(const float* __restrict__ dY,
                                                                     float* __restrict__ dIn,
                                                                     const float* __restrict__ mask,
                                                                     long long rows, int C, Shortcut sc,
                                                                     long long total) {
  const long long idx = (long long)blockIdx.x * kThreads + threadIdx.x;
  if (idx >= total) return;
  const int words = sc.Cs / 4;
  const int c = (int)(idx % words) * 4;
  long long m = idx / words;
  const int k = (int)(m / rows);
  m -= (long long)k * rows;
  const int j = (int)(m % sc.W), i = (int)((m / sc.W) % sc.H);
  const long long b = m / ((long long)sc.W * sc.H);
  const long long at = k * sc.stride + ((b * (sc.st * sc.H) + sc.st * i) * (sc.st * sc.W) + sc.st * j) * sc.Cs + c;
  f32x4 g = *reinterpret_cast<const f32x4*>(dY + ((long long)k * rows + m) * C + c);
  if (mask != nullptr) {
    const f32x4 keep = *reinterpret_cast<const f32x4*>(mask + at);
#pragma unroll
    for (int r = 0; r < 4; ++r)
      if (!(keep[r] > 0.f)) g[r] = 0.f;
  }
  *reinterpret_cast<f32x4*>(dIn + at) += g;
}

// dst[k][b][i][j][c] = src[k][b][2 i][2 j][c]: the pixels a stride-2 1x1 convolution reads, as a
// dense matrix [K][B H W][C].  One thread per 16-byte word of dst.
__global__ __launch_bounds__(kThreads) void subsample2_kernel(const float* __restrict__ src,
                                                              float* __restrict__ dst, long long images,
                                                              int H, int W, int C, long long total) {
  const long long idx = (long long)blockIdx.x * kThreads + threadIdx.x;
  if (idx >= total) return;
  const int words = C / 4;
  const int c = (int)(idx % words) * 4;
  long long m = idx / words;
  const int j = (int)(m % W);
  m /= W;
  const int i = (int)(m % H);
  const long long img = m / H;
  const long long at = ((img * (2 * H) + 2 * i) * (2 * W) + 2 * j) * C + c;
  *reinterpret_cast<f32x4*>(dst + idx * 4) = *reinterpret_cast<const f32x4*>(src + at);
}

// dst += src, element by element (n a multiple of 4, both 16-byte aligned).
__global__ __launch_bounds__(kThreads) void add_into_kernel(float* __restrict__ dst,
                                                            const float* __restrict__ src, long long words) {
  const long long idx = (long long)blockIdx.x * kThreads + threadIdx.x;
  if (idx >= words) return;
  *reinterpret_cast<f32x4*>(dst + idx * 4) += *reinterpret_cast<const f32x4*>(src + idx * 4);
}

// Global average pooling: P[k][b][c] = mean over the H W positions of A[k][b][.][.][c] (summed
// in position order), P rows of pitch ldp; and its backward pass fused with the ReLU the image
// came from: dA[k][b][i][j][c] = dP[k][b][c] / (H W) where A > 0 (mask null: everywhere).
__global__ __launch_bounds__(kThreads) void avgpool_kernel(const float* __restrict__ A, float* __restrict__ P,
                                                           long long images, int HW, int C, int ldp) {
  const long long idx = (long long)blockIdx.x * kThreads + threadIdx.x;
  const int words = C / 4;
  if (idx >= images * words) return;
  const int c = (int)(idx % words) * 4;
  const long long img = idx / words;
  const float* a = A + img * (long long)HW * C + c;
  f32x4 acc = {0.f, 0.f, 0.f, 0.f};
  for (int p = 0; p < HW; ++p) acc += *reinterpret_cast<const f32x4*>(a + (long long)p * C);
  const float inv = 1.f / (float)HW;
  *reinterpret_cast<f32x4*>(P + img * ldp + c) = acc * inv;
}
__global__ __launch_bounds__(kThreads) void avgpool_backward_kernel(const float* __restrict__ dP,
                                                                    const float* __restrict__ mask,
                                                                    float* __restrict__ dA, long long images,
                                                                    int HW, int C, int ldp) {
  const long long idx = (long long)blockIdx.x * kThreads + threadIdx.x;
  const int words = C / 4;
  if (idx >= images * HW * words) return;
  const int c = (int)(idx % words) * 4;
  const long long img = idx / words / HW;
  f32x4 g = *reinterpret_cast<const f32x4*>(dP + img * ldp + c) * (1.f / (float)HW);
  if (mask != nullptr) {
    const f32x4 keep = *reinterpret_cast<const f32x4*>(mask + idx * 4);
#pragma unroll
    for (int r = 0; r < 4; ++r)
      if (!(keep[r] > 0.f)) g[r] = 0.f;
  }
  *reinterpret_cast<f32x4*>(dA + idx * 4) = g;
}

// Chunk sums for the backward pass: part[k][chunk][0..C) = sum dY Xh, [C..2C) = sum dY, with
// Xh = (Z - mean) inv_std recomputed from Z.
__global__ __launch_bounds__(kThreads) void bn_backward_partial_kernel(const float* __restrict__ Z,
                                                                       const float* __restrict__ dY,
                                                                       const float* __restrict__ stats,
                                                                       float* __restrict__ part,
                                                                       long long rows, int C, int chunks,
                                                                       int chunk_rows) {
  __shared__ f32x4 buf[kThreads];
  const ChunkThread t = chunk_thread(rows, C, chunk_rows);
  const int k = blockIdx.y;
  const long long base = ((long long)k * rows) * C + 4 * t.cw;
  f32x4 sg = {0.f, 0.f, 0.f, 0.f}, sb = {0.f, 0.f, 0.f, 0.f};
  if (t.live) {
    const f32x4 mu = *reinterpret_cast<const f32x4*>(stats + ((long long)k * 2) * C + 4 * t.cw);
    const f32x4 inv = *reinterpret_cast<const f32x4*>(stats + ((long long)k * 2 + 1) * C + 4 * t.cw);
    for (long long r = t.r0 + t.grp; r < t.r1; r += 16) {
      const f32x4 dy = *reinterpret_cast<const f32x4*>(dY + base + r * C);
      const f32x4 xh = (*reinterpret_cast<const f32x4*>(Z + base + r * C) - mu) * inv;
      sg += dy * xh;
      sb += dy;
    }
  }
  const f32x4 tg = combine_groups(sg, t, buf);
  const f32x4 tb = combine_groups(sb, t, buf);
  if (t.live && t.grp == 0) {
    float* dst = part + ((long long)k * chunks + blockIdx.x) * 2 * C + 4 * t.cw;
    *reinterpret_cast<f32x4*>(dst) = tg;
    *reinterpret_cast<f32x4*>(dst + C) = tb;
  }
}

// dZ = gamma inv_std (dY - dbeta / N - Xh dgamma / N), written to dZ, which may be dY itself or Z
// (every thread reads its own word of both before it writes).
__global__ __launch_bounds__(kThreads) void bn_backward_apply_kernel(
    const float* Z, const float* dY, float* dZ, const float* __restrict__ stats,
    const float* __restrict__ params, const float* __restrict__ grad, long long strideParams,
    long long gam_off, long long bet_off, long long rows, int C, long long total) {
  const long long idx = (long long)blockIdx.x * kThreads + threadIdx.x;
  if (idx >= total) return;
  const int words = C / 4;
  const int c = (int)(idx % words) * 4;
  const int k = (int)(idx / words / rows);
  const f32x4 mu = *reinterpret_cast<const f32x4*>(stats + ((long long)k * 2) * C + c);
  const f32x4 inv = *reinterpret_cast<const f32x4*>(stats + ((long long)k * 2 + 1) * C + c);
  const f32x4 ga = *reinterpret_cast<const f32x4*>(params + k * strideParams + gam_off + c);
  const f32x4 dga = *reinterpret_cast<const f32x4*>(grad + k * strideParams + gam_off + c);
  const f32x4 dbe = *reinterpret_cast<const f32x4*>(grad + k * strideParams + bet_off + c);
  const float inv_n = 1.f / (float)rows;
  const f32x4 xh = (*reinterpret_cast<const f32x4*>(Z + idx * 4) - mu) * inv;
  const f32x4 dy = *reinterpret_cast<const f32x4*>(dY + idx * 4);
  *reinterpret_cast<f32x4*>(dZ + idx * 4) = ga * inv * (dy - dbe * inv_n - xh * (dga * inv_n));
}

unsigned blocks_for(long long total) { return (unsigned)((total + kThreads - 1) / kThreads); }

}  // namespace

int launch_unfold3x3(const float* X, int64_t strideX, float* col, int64_t strideCol, int ld, int K,
                     int B, int H, int W, int C, int stride, hipStream_t s) {
  ImgShape sh{H, W, C, ld, (long long)B * H * W, 0, stride};
  sh.total = (long long)K * sh.rows * (ld / 4);
  if (ld % 4 || ld < 9 * C || sh.total <= 0 || sh.total >= (1ll << 31) * kThreads || stride < 1 || stride > 2)
    return -1;
  if (C % 4 == 0)
    unfold3x3_kernel<true><<<blocks_for(sh.total), kThreads, 0, s>>>(X, col, sh, strideX, strideCol);
  else
    unfold3x3_kernel<false><<<blocks_for(sh.total), kThreads, 0, s>>>(X, col, sh, strideX, strideCol);
  return 0;
}

int launch_fold3x3(const float* dcol, int64_t strideCol, int ld, float* dX, const float* mask,
                   int64_t strideX, int K, int B, int H, int W, int C, int stride, hipStream_t s) {
  ImgShape sh{H, W, C, ld, (long long)B * H * W * stride * stride, 0, stride};
  sh.total = (long long)K * sh.rows * (C / 4);
  if (C % 4 || ld < 9 * C || sh.total <= 0 || sh.total >= (1ll << 31) * kThreads || stride < 1 || stride > 2)
    return -1;
  fold3x3_kernel<<<blocks_for(sh.total), kThreads, 0, s>>>(dcol, dX, mask, sh, strideCol, strideX);
  return 0;
}

void launch_flip_filters(const float* W, int64_t strideW, int ldw, float* Wt, int K, int Cout, int Cin,
                         hipStream_t s) {
  const int cblocks = (Cin + 31) / 32;
  flip_filters_kernel<<<dim3((unsigned)(Cout / 32 * cblocks), 9u, (unsigned)K), kThreads, 0, s>>>(
      W, strideW, ldw, Wt, Cout, Cin, cblocks);
}

bool first_conv_fits(int C, int Cout, int64_t rows) {
  return C >= 1 && C <= 3 && Cout % 32 == 0 && Cout <= 256 && rows < (1 << 24);
}

int first_conv_chunks(int64_t rows) { return (int)((rows + kFirstChunk - 1) / kFirstChunk); }

static FirstConv first_shape(int H, int W, int Cout, int64_t rows, int64_t strideParams, int ldw) {
  return FirstConv{H, W, Cout, 1.f / (float)W, 1.f / (float)H, rows, strideParams, ldw};
}

int launch_first_conv_forward(const float* X, const float* params, int64_t strideParams, int64_t w_off,
                              int64_t b_off, int ldw, float* out, int relu, int round, int K,
                              int64_t rows, int H, int W, int C, int Cout, hipStream_t s) {
  if (!first_conv_fits(C, Cout, rows)) return -1;
  const FirstConv f = first_shape(H, W, Cout, rows, strideParams, ldw);
  const dim3 grid((unsigned)((rows + 127) / 128), (unsigned)K);
  const size_t lds = (size_t)Cout * 33 * 4;
  if (C == 1) first_conv_forward_kernel<1><<<grid, kThreads, lds, s>>>(X, params, w_off, b_off, out, f, relu, round);
  else if (C == 2) first_conv_forward_kernel<2><<<grid, kThreads, lds, s>>>(X, params, w_off, b_off, out, f, relu, round);
  else first_conv_forward_kernel<3><<<grid, kThreads, lds, s>>>(X, params, w_off, b_off, out, f, relu, round);
  return 0;
}

int launch_first_conv_wgrad(const float* X, const float* dout, float* partial, float* grad,
                            int64_t strideParams, int64_t w_off, int64_t b_off, int ldw, int round,
                            int skip_bias, int K, int64_t rows, int H, int W, int C, int Cout,
                            double* sumsq, int64_t sumsq_stride, hipStream_t s) {
  if (!first_conv_fits(C, Cout, rows)) return -1;
  const FirstConv f = first_shape(H, W, Cout, rows, strideParams, ldw);
  const int chunks = first_conv_chunks(rows);
  const dim3 grid((unsigned)chunks, (unsigned)K);
  if (C == 1) first_conv_wgrad_kernel<1><<<grid, kThreads, 0, s>>>(X, dout, partial, chunks, f, round);
  else if (C == 2) first_conv_wgrad_kernel<2><<<grid, kThreads, 0, s>>>(X, dout, partial, chunks, f, round);
  else first_conv_wgrad_kernel<3><<<grid, kThreads, 0, s>>>(X, dout, partial, chunks, f, round);
  first_conv_wgrad_finish_kernel<<<dim3((unsigned)(Cout / 2), (unsigned)K), 1024, 0, s>>>(
      partial, chunks, C, grad, w_off, b_off, sumsq, sumsq_stride, f, skip_bias);
  return Cout / 2;     // sum-of-squares slots written per replica
}

int bn_chunks(int64_t rows, int C, int K) { return chunk_plan(rows, C, K).chunks; }

int launch_bn_stats(const float* Z, float* scratch, float* stats, int K, int64_t rows, int C, float eps,
                    hipStream_t s) {
  if (C % 4 || C < 4 || C > 4 * kThreads || rows < 1) return -1;
  const ChunkPlan pl = chunk_plan(rows, C, K);
  const int chunks = pl.chunks;
  float* pmean = scratch;
  float* pm2 = scratch + (long long)K * chunks * C;
  bn_stats_partial_kernel<<<dim3((unsigned)chunks, (unsigned)K, (unsigned)pl.col_blocks), kThreads, 0, s>>>(
      Z, pmean, pm2, rows, C, chunks, pl.chunk_rows);
  bn_stats_finish_kernel<<<dim3((unsigned)((C + 63) / 64), (unsigned)K), 64 * kBnChains, 0, s>>>(
      pmean, pm2, stats, rows, C, chunks, pl.chunk_rows, eps);
  return 0;
}

int launch_add_into(float* dst, const float* src, int64_t n, hipStream_t s) {
  if (n < 4 || n % 4) return -1;
  add_into_kernel<<<blocks_for(n / 4), kThreads, 0, s>>>(dst, src, n / 4);
  return 0;
}

int launch_subsample2(const float* src, float* dst, int64_t images, int H, int W, int C, hipStream_t s) {
  if (C % 4 || C < 4 || H < 1 || W < 1 || images < 1) return -1;
  const long long total = images * H * W * (C / 4);
  subsample2_kernel<<<blocks_for(total), kThreads, 0, s>>>(src, dst, images, H, W, C, total);
  return 0;
}

int launch_bn_forward(const float* Z, float* scratch, float* stats, const float* params,
                      int64_t strideParams, int64_t gam_off, int64_t bet_off, float* out, int K,
                      int64_t rows, int C, float eps, const ShortcutDesc* shortcut, hipStream_t s) {
  if (C % 4 || C < 4 || C > 4 * kThreads || rows < 1) return -1;
  Shortcut sc{nullptr, 0, 1, 1, 0, 1, nullptr, nullptr, 0, 0};
  if (shortcut != nullptr && shortcut->pz != nullptr) {
    if (shortcut->pstats == nullptr) return -1;
    sc.pz = shortcut->pz; sc.pstats = shortcut->pstats;
    sc.pgam_off = shortcut->pgam_off; sc.pbet_off = shortcut->pbet_off;
  } else if (shortcut != nullptr) {
    if (shortcut->Cs % 4 || shortcut->Cs > C || shortcut->H < 1 || shortcut->W < 1 ||
        rows % ((int64_t)shortcut->H * shortcut->W) || shortcut->step < 1 || shortcut->step > 2)
      return -1;
    sc = Shortcut{shortcut->src, shortcut->stride, shortcut->H, shortcut->W, shortcut->Cs, shortcut->step,
                  nullptr, nullptr, 0, 0};
  }
  const ChunkPlan pl = chunk_plan(rows, C, K);
  const int chunks = pl.chunks;
  float* pmean = scratch;
  float* pm2 = scratch + (long long)K * chunks * C;
  bn_stats_partial_kernel<<<dim3((unsigned)chunks, (unsigned)K, (unsigned)pl.col_blocks), kThreads, 0, s>>>(
      Z, pmean, pm2, rows, C, chunks, pl.chunk_rows);
  bn_stats_finish_kernel<<<dim3((unsigned)((C + 63) / 64), (unsigned)K), 64 * kBnChains, 0, s>>>(
      pmean, pm2, stats, rows, C, chunks, pl.chunk_rows, eps);
  const long long total = (long long)K * rows * (C / 4);
  bn_apply_kernel<<<blocks_for(total), kThreads, 0, s>>>(Z, stats, params, strideParams, gam_off, bet_off,
                                                        out, rows, C, total, sc);
  return 0;
}

int launch_shortcut_backward(const float* dY, float* dIn, const float* mask, const ShortcutDesc& d, int K,
                             int64_t rows, int C, hipStream_t s) {
  if (d.Cs % 4 || d.Cs > C || d.Cs < 4 || rows % ((int64_t)d.H * d.W) || d.step < 1 || d.step > 2) return -1;
  const Shortcut sc{nullptr, d.stride, d.H, d.W, d.Cs, d.step, nullptr, nullptr, 0, 0};
  const long long total = (long long)K * rows * (d.Cs / 4);
  shortcut_backward_kernel<<<blocks_for(total), kThreads, 0, s>>>(dY, dIn, mask, rows, C, sc, total);
  return 0;
}

int launch_avgpool(const float* A, float* P, int64_t images, int HW, int C, int ldp, hipStream_t s) {
  if (C % 4 || HW < 1 || ldp < C || ldp % 4) return -1;
  avgpool_kernel<<<blocks_for(images * (C / 4)), kThreads, 0, s>>>(A, P, images, HW, C, ldp);
  return 0;
}

int launch_avgpool_backward(const float* dP, const float* mask, float* dA, int64_t images, int HW, int C,
                            int ldp, hipStream_t s) {
  if (C % 4 || HW < 1 || ldp < C || ldp % 4) return -1;
  avgpool_backward_kernel<<<blocks_for(images * HW * (C / 4)), kThreads, 0, s>>>(dP, mask, dA, images, HW, C, ldp);
  return 0;
}

int launch_bn_backward_partials(const float* Z, const float* dY, const float* stats, float* part, int K,
                                int64_t rows, int C, hipStream_t s) {
  if (C % 4 || C < 4 || C > 4 * kThreads || rows < 1) return -1;
  const ChunkPlan pl = chunk_plan(rows, C, K);
  bn_backward_partial_kernel<<<dim3((unsigned)pl.chunks, (unsigned)K, (unsigned)pl.col_blocks), kThreads, 0,
                               s>>>(Z, dY, stats, part, rows, C, pl.chunks, pl.chunk_rows);
  return pl.chunks;
}

void launch_bn_backward_apply(const float* Z, const float* dY, float* dZ, const float* stats,
                              const float* params, const float* grad, int64_t strideParams,
                              int64_t gam_off, int64_t bet_off, int K, int64_t rows, int C, hipStream_t s) {
  const long long total = (long long)K * rows * (C / 4);
  bn_backward_apply_kernel<<<blocks_for(total), kThreads, 0, s>>>(Z, dY, dZ, stats, params, grad, strideParams,
                                                                 gam_off, bet_off, rows, C, total);
}

int colsum_chunks(int64_t rows, int N, int K) { return chunk_plan(rows, N, K).chunks; }

int launch_colsum_partials(const float* A, int64_t rows, int N, int K, float* partial, hipStream_t s) {
  if (N % 4 || N < 4 || N > 4 * kThreads || rows < 1) return -1;
  const ChunkPlan pl = chunk_plan(rows, N, K);
  colsum_partial_kernel<<<dim3((unsigned)pl.chunks, (unsigned)K, (unsigned)pl.col_blocks), kThreads, 0, s>>>(
      A, partial, rows, N, pl.chunks, pl.chunk_rows);
  return pl.chunks;
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
