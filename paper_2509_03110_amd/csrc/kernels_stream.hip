// Streaming kernels of the update path: gradient-norm reduction, ascent perturbation,
// descent + coupling, center update.  All are HBM-bandwidth bound: every array is touched
// once per kernel with 128-bit accesses, consecutive lanes on consecutive 16-byte words.
#include <type_traits>

#include "engine.h"

namespace lsam {
namespace {

constexpr int kThreads = 256;

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef unsigned short u16x4 __attribute__((ext_vector_type(4)));

template <int VEC> struct Vec;
template <> struct Vec<4> { typedef f32x4 type; };
template <> struct Vec<1> { typedef float type; };

template <int VEC>
__device__ __forceinline__ typename Vec<VEC>::type ldv(const float* p) {
  return __builtin_nontemporal_load(reinterpret_cast<const typename Vec<VEC>::type*>(p));
}
template <int VEC>
__device__ __forceinline__ void stv(float* p, typename Vec<VEC>::type v) {
  __builtin_nontemporal_store(v, reinterpret_cast<typename Vec<VEC>::type*>(p));
}
// Parameters that the next kernels read back: streamed past the caches when all replicas
// together are far larger than they are (K d floats; measured at 3.2 GB: +5-9 % for the two
// kernels with streaming stores), left in them when they fit (at 67 MB the following forward
// GEMMs and the next descent find them there: -2 % per step).
constexpr int64_t kCacheResidentBytes = 96ll << 20;
template <int VEC, bool STREAM>
__device__ __forceinline__ void st_param(float* p, typename Vec<VEC>::type v) {
  if constexpr (STREAM) __builtin_nontemporal_store(v, reinterpret_cast<typename Vec<VEC>::type*>(p));
  else *reinterpret_cast<typename Vec<VEC>::type*>(p) = v;
}
// y / g'_prev are re-read by later kernels and other replicas: ordinary cached access.
template <int VEC>
__device__ __forceinline__ typename Vec<VEC>::type ldc(const float* p) {
  return *reinterpret_cast<const typename Vec<VEC>::type*>(p);
}

__device__ __forceinline__ float elem(const f32x4& v, int i) { return v[i]; }
__device__ __forceinline__ float elem(const float& v, int) { return v; }
__device__ __forceinline__ void set_elem(f32x4& v, int i, float a) { v[i] = a; }
__device__ __forceinline__ void set_elem(float& v, int, float a) { v = a; }

__device__ __forceinline__ unsigned short bf16_bits(float f) {
  return __builtin_bit_cast(unsigned short, static_cast<__bf16>(f));
}
template <int VEC>
__device__ __forceinline__ void store_bf16(uint16_t* p, const typename Vec<VEC>::type& v) {
  if constexpr (VEC == 4) {
    u16x4 o;
#pragma unroll
    for (int i = 0; i < 4; ++i) o[i] = bf16_bits(v[i]);
    // Plain store: a wavefront's 64-byte pieces of neighbouring blocks merge in L2 before they
    // go out; the streaming hint measured no better once the copy became blocked.
    *reinterpret_cast<u16x4*>(p) = o;
  } else {
    *p = bf16_bits(v);
  }
}

__device__ __forceinline__ double wave_sum(double v) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) v += __shfl_down(v, off, 64);
  return v;
}

// Sum over the block in a fixed order; result valid in thread 0.
__device__ __forceinline__ double block_sum(double v) {
  __shared__ double part[kThreads / 64];
  v = wave_sum(v);
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  if (lane == 0) part[wave] = v;
  __syncthreads();
  double r = 0.0;
  if (threadIdx.x == 0) {
#pragma unroll
    for (int w = 0; w < kThreads / 64; ++w) r += part[w];
  }
  __syncthreads();
  return r;
}

// ---- gradient norm, pass 1 ------------------------------------------------------------------
template <int VEC>
__global__ __launch_bounds__(kThreads) void sumsq_partials_kernel(
    const float* __restrict__ g, int64_t g_stride, int64_t nv, double* __restrict__ partials,
    int nblk) {
  const int k = blockIdx.y;
  const int64_t chunk = (nv + nblk - 1) / nblk;
  const int64_t beg = (int64_t)blockIdx.x * chunk;
  const int64_t end = beg + chunk < nv ? beg + chunk : nv;
  const float* gk = g + (int64_t)k * g_stride;
  float a0 = 0.f, a1 = 0.f, a2 = 0.f, a3 = 0.f;
  int64_t i = beg + threadIdx.x;
  for (; i + 3 * kThreads < end; i += 4 * kThreads) {
    auto v0 = ldv<VEC>(gk + i * VEC);
    auto v1 = ldv<VEC>(gk + (i + kThreads) * VEC);
    auto v2 = ldv<VEC>(gk + (i + 2 * kThreads) * VEC);
    auto v3 = ldv<VEC>(gk + (i + 3 * kThreads) * VEC);
#pragma unroll
    for (int e = 0; e < VEC; ++e) {
      a0 += elem(v0, e) * elem(v0, e);
      a1 += elem(v1, e) * elem(v1, e);
      a2 += elem(v2, e) * elem(v2, e);
      a3 += elem(v3, e) * elem(v3, e);
    }
  }
  for (; i < end; i += kThreads) {
    auto v0 = ldv<VEC>(gk + i * VEC);
#pragma unroll
    for (int e = 0; e < VEC; ++e) a0 += elem(v0, e) * elem(v0, e);
  }
  double s = ((double)a0 + (double)a1) + ((double)a2 + (double)a3);
  s = block_sum(s);
  if (threadIdx.x == 0) partials[(int64_t)k * nblk + blockIdx.x] = s;
}

// ---- gradient norm of a dense layer's weight gradient from two Gram matrices ---------------------
// ||dZ^T A||_F^2 = sum_{b,b'} (dZ dZ^T)[b,b'] (A A^T)[b,b']: the squared norm of the weight
// gradient dW = dZ^T A [out x in] of a layer with batch B is the inner product of the two B x B
// Gram matrices of its factors, which take 2 B^2 (out + in) flops instead of 2 B out in.  This
// kernel is the inner product: partial sums in the fixed order of sumsq_partials_kernel.  Each
// Gram matrix may arrive as several partial matrices (its contraction split over workgroups),
// `piece_stride` elements apart, which are added up first, in order.
__device__ __forceinline__ f32x4 gram_word(const float* p, int64_t i, int pieces, int64_t piece_stride) {
  f32x4 u = ldc<4>(p + i * 4);
  for (int j = 1; j < pieces; ++j) {
    const f32x4 t = ldc<4>(p + (int64_t)j * piece_stride + i * 4);
#pragma unroll
    for (int e = 0; e < 4; ++e) u[e] += t[e];
  }
  return u;
}

__global__ __launch_bounds__(kThreads) void gram_dot_partials_kernel(
    const float* __restrict__ G1, const float* __restrict__ G2, int64_t stride, int64_t nv, int pieces1,
    int pieces2, int64_t piece_stride, double* __restrict__ partials, int64_t pstride, int nblk) {
  const int k = blockIdx.y;
  const int64_t chunk = (nv + nblk - 1) / nblk;
  const int64_t beg = (int64_t)blockIdx.x * chunk;
  const int64_t end = beg + chunk < nv ? beg + chunk : nv;
  const float* a = G1 + (int64_t)k * stride;
  const float* b = G2 + (int64_t)k * stride;
  float a0 = 0.f, a1 = 0.f;
  int64_t i = beg + threadIdx.x;
  for (; i + kThreads < end; i += 2 * kThreads) {
    const auto u0 = gram_word(a, i, pieces1, piece_stride), w0 = gram_word(b, i, pieces2, piece_stride);
    const auto u1 = gram_word(a, i + kThreads, pieces1, piece_stride);
    const auto w1 = gram_word(b, i + kThreads, pieces2, piece_stride);
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      a0 += u0[e] * w0[e];
      a1 += u1[e] * w1[e];
    }
  }
  for (; i < end; i += kThreads) {
    const auto u0 = gram_word(a, i, pieces1, piece_stride), w0 = gram_word(b, i, pieces2, piece_stride);
#pragma unroll
    for (int e = 0; e < 4; ++e) a0 += u0[e] * w0[e];
  }
  const double s = block_sum((double)a0 + (double)a1);
  if (threadIdx.x == 0) partials[(int64_t)k * pstride + blockIdx.x] = s;
}

// ---- gradient norm, pass 2 (+ mean loss) ----------------------------------------------------
__global__ __launch_bounds__(kThreads) void norm_finish_kernel(
    const double* __restrict__ partials, int nblk, int64_t pstride, float rho, float gamma,
    float* __restrict__ norms, float* __restrict__ scale, const float* __restrict__ loss_rows,
    int B, float* __restrict__ loss_out, int32_t* __restrict__ restart) {
  const int k = blockIdx.x;
  if (restart != nullptr && threadIdx.x == 0) {     // 2 (sum just served) -> 1 (restart it in this step) -> 0
    const int32_t m = restart[k];
    if (m > 0) restart[k] = m - 1;
  }
  double s = 0.0;
  for (int i = threadIdx.x; i < nblk; i += kThreads) s += partials[(int64_t)k * pstride + i];
  s = block_sum(s);
  if (threadIdx.x == 0) {
    const double n = sqrt(s);
    norms[k] = (float)n;
    scale[k] = (float)((double)rho / (n + (double)gamma));
  }
  if (loss_rows != nullptr && loss_out != nullptr) {
    double l = 0.0;
    for (int i = threadIdx.x; i < B; i += kThreads) l += (double)loss_rows[(int64_t)k * B + i];
    l = block_sum(l);
    if (threadIdx.x == 0) loss_out[k] = (float)(l / (double)B);
  }
}

// ---- ascent perturbation ----------------------------------------------------------------------
// BF16_OUT: x~ exists only as the bf16 operand copy of the weight matrices (blocked layout);
// elements that belong to no weight matrix (biases, padding) are not stored at all -- the
// perturbed biases are formed in the GEMM epilogue from x, g1 and scale.
template <int VEC, bool BF16_OUT, bool STREAM>
__global__ __launch_bounds__(kThreads) void perturb_kernel(
    const float* __restrict__ x, const float* __restrict__ g, int64_t g_stride,
    const float* __restrict__ scale, float* __restrict__ xt, uint16_t* __restrict__ xt16,
    ShadowMap map, int64_t shadow_stride, int64_t stride, int64_t nv) {
  const int k = blockIdx.y;
  const int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x;
  if (i >= nv) return;
  int64_t so = 0;
  if constexpr (BF16_OUT) {
    so = shadow_offset4(map, i * VEC);
    if (so < 0) return;
  }
  const float sc = scale[k];
  auto xv = ldv<VEC>(x + (int64_t)k * stride + i * VEC);
  auto gv = ldv<VEC>(g + (int64_t)k * g_stride + i * VEC);
  typename Vec<VEC>::type o;
#pragma unroll
  for (int e = 0; e < VEC; ++e) set_elem(o, e, ascent_point(elem(xv, e), sc, elem(gv, e)));
  if constexpr (BF16_OUT) {
    store_bf16<VEC>(xt16 + (int64_t)k * shadow_stride + so, o);
  } else {
    st_param<VEC, STREAM>(xt + (int64_t)k * stride + i * VEC, o);
  }
}

// The same for bf16 operands, walking the weight matrices in tiles instead of the flat vector: a
// workgroup takes 8 rows x 128 columns of one matrix, a wavefront 8 rows x 32 columns, so that the
// wavefront's 256 results are 512 consecutive bytes of one block of the copy (the flat walk
// writes 64-byte pieces of 8 different blocks per wavefront and reached 67 % of HBM peak here
// against 80 % for the fp32 kernel) while x and g1 are still read in 512-byte row pieces.
struct TileMap {
  int32_t n;
  int32_t first[LSAM_MAX_LAYERS + 1];   // first workgroup of each matrix; [n] = total
  int32_t ctiles[LSAM_MAX_LAYERS];      // 128-column tiles per row of W_l
  int32_t rows[LSAM_MAX_LAYERS];
};

__global__ __launch_bounds__(kThreads) void perturb_tiled_kernel(
    const float* __restrict__ x, const float* __restrict__ g, int64_t g_stride,
    const float* __restrict__ scale, uint16_t* __restrict__ xt16, ShadowMap map, TileMap tiles,
    int64_t shadow_stride, int64_t stride) {
  const int k = blockIdx.y;
  int s = 0;
  while (s + 1 < tiles.n && (int)blockIdx.x >= tiles.first[s + 1]) ++s;
  const int t = blockIdx.x - tiles.first[s];
  const int rg = t / tiles.ctiles[s], ct = t - rg * tiles.ctiles[s];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int r = rg * 8 + (lane >> 3);
  const int c = ct * 128 + wave * 32 + (lane & 7) * 4;
  if (r >= tiles.rows[s] || c >= map.ldw[s]) return;
  const int64_t flat = map.begin[s] + (int64_t)r * map.ldw[s] + c;
  const float sc = scale[k];
  const auto xv = ldv<4>(x + (int64_t)k * stride + flat);
  const auto gv = ldv<4>(g + (int64_t)k * g_stride + flat);
  typename Vec<4>::type o;
#pragma unroll
  for (int e = 0; e < 4; ++e) set_elem(o, e, ascent_point(elem(xv, e), sc, elem(gv, e)));
  store_bf16<4>(xt16 + (int64_t)k * shadow_stride + map.shadow[s] + b32s_offset(r, c, map.cblocks[s]), o);
}

// ---- descent + coupling -------------------------------------------------------------------------
// One workgroup updates 256 vector words of one replica; consecutive workgroups take the same
// words of the K replicas in turn, so the K readers of a piece of y run close together and y
// comes from HBM once.  (Looping over the replicas inside one thread, which reads y exactly
// once, measured 8-12 % slower at K = 8 and 16; sending the K workgroups of a piece to the same
// XCD, so that y misses only one L2, measured 4-9 % slower: the other XCDs' misses are served
// by the memory-side cache, and the launch order here keeps each XCD on fewer DRAM pages.)
template <int VEC, bool SHADOW, bool STREAM, typename NOISE>
__global__ __launch_bounds__(kThreads) void descent_kernel(
    float* __restrict__ x, const float* __restrict__ g, int64_t g_stride, float* __restrict__ v,
    float* __restrict__ S, const float* __restrict__ y, uint16_t* __restrict__ shadow,
    ShadowMap map, int64_t shadow_stride, int64_t stride, int64_t nv, int K, ReplicaScalars lam,
    float lr, float mu, int nesterov, NOISE noise, const int32_t* __restrict__ restart) {
  const int64_t b = blockIdx.x;
  const int k = (int)(b % K);
  const int64_t i = (b / K) * kThreads + threadIdx.x;
  if (i >= nv) return;
  const auto yv = ldc<VEC>(y + i * VEC);
  const int64_t o = (int64_t)k * stride + i * VEC;
  auto xv = ldv<VEC>(x + o);
  auto gv = ldv<VEC>(g + (int64_t)k * g_stride + i * VEC);
  auto vv = ldv<VEC>(v + o);
  typename Vec<VEC>::type sv;
  if (restart != nullptr && restart[k] == 1) {       // the sum starts afresh: its memory is stale
#pragma unroll
    for (int e = 0; e < VEC; ++e) set_elem(sv, e, 0.f);
  } else {
    sv = ldv<VEC>(S + o);
  }
  const float lk = lam.v[k];
  float xi[4] = {0.f, 0.f, 0.f, 0.f};      // sigma sqrt(2 eta) xi of the Langevin sampler
  if constexpr (!std::is_same<NOISE, NoNoise>::value) {
    if constexpr (VEC == 4) {
      langevin4(noise, k, i * 4, xi);
    } else {
      float grp[4];
      langevin4(noise, k, i & ~(int64_t)3, grp);
      xi[0] = grp[i & 3];
    }
  }
#pragma unroll
  for (int e = 0; e < VEC; ++e) {
    float xe = elem(xv, e), ve = elem(vv, e), se = elem(sv, e);
    sampler_step(elem(gv, e), elem(yv, e), lk, lr, mu, nesterov, xi[e], xe, ve, se);
    set_elem(vv, e, ve);
    set_elem(xv, e, xe);
    set_elem(sv, e, se);
  }
  st_param<VEC, STREAM>(x + o, xv);
  stv<VEC>(v + o, vv);
  stv<VEC>(S + o, sv);
  if constexpr (SHADOW) {
    const int64_t so = shadow_offset4(map, i * VEC);
    if (so >= 0) store_bf16<VEC>(shadow + (int64_t)k * shadow_stride + so, xv);
  }
}

// ---- average over replicas (synchronous data-parallel baseline) ---------------------------------
template <int VEC>
__global__ __launch_bounds__(kThreads) void grad_mean_kernel(
    const float* src, int64_t src_stride, float* dst, int64_t dst_stride, int64_t nv, int K,
    int copies) {
  const int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x;
  if (i >= nv) return;
  auto acc = ldv<VEC>(src + i * VEC);
  for (int k = 1; k < K; ++k) {
    const auto gv = ldv<VEC>(src + (int64_t)k * src_stride + i * VEC);
#pragma unroll
    for (int e = 0; e < VEC; ++e) set_elem(acc, e, elem(acc, e) + elem(gv, e));
  }
  const float inv = 1.f / (float)K;
#pragma unroll
  for (int e = 0; e < VEC; ++e) set_elem(acc, e, elem(acc, e) * inv);
  for (int c = 0; c < copies; ++c) stv<VEC>(dst + (int64_t)c * dst_stride + i * VEC, acc);
}

// ---- center update ------------------------------------------------------------------------------
template <int VEC>
__global__ __launch_bounds__(kThreads) void center_kernel(
    float* __restrict__ S, float* __restrict__ y, float* __restrict__ gprev, int64_t stride,
    int64_t nv, DueList due, float inv_m, float beta, float lr_center, int has_prev,
    int32_t* __restrict__ restart) {
  // (no thread of this kernel reads a mark: a replica that is due has taken a step since it
  // was last served, and that step's norm kernel had counted its mark down to at most 1)
  if (restart != nullptr && blockIdx.x == 0 && (int)threadIdx.x < due.n) restart[due.idx[threadIdx.x]] = 2;
  const int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x;
  if (i >= nv) return;
  typename Vec<VEC>::type tot, zero;
#pragma unroll
  for (int e = 0; e < VEC; ++e) { set_elem(tot, e, 0.f); set_elem(zero, e, 0.f); }
  for (int j = 0; j < due.n; ++j) {
    float* p = S + (int64_t)due.idx[j] * stride + i * VEC;
    auto sv = ldv<VEC>(p);
#pragma unroll
    for (int e = 0; e < VEC; ++e) set_elem(tot, e, elem(tot, e) + elem(sv, e));
    if (restart == nullptr) stv<VEC>(p, zero);
  }
  auto yv = ldc<VEC>(y + i * VEC);
  auto pv = ldc<VEC>(gprev + i * VEC);
  typename Vec<VEC>::type gp;
#pragma unroll
  for (int e = 0; e < VEC; ++e) {
    const float gpe = elem(tot, e) * inv_m - elem(yv, e);
    const float ge = has_prev ? gpe + beta * (gpe - elem(pv, e)) : gpe;
    set_elem(gp, e, gpe);
    set_elem(yv, e, elem(yv, e) + lr_center * ge);
  }
  *reinterpret_cast<typename Vec<VEC>::type*>(y + i * VEC) = yv;
  *reinterpret_cast<typename Vec<VEC>::type*>(gprev + i * VEC) = gp;
}

// ---- small utility kernels ------------------------------------------------------------------------
template <int VEC>
__global__ __launch_bounds__(kThreads) void broadcast_kernel(
    const float* __restrict__ src, float* __restrict__ dst, int64_t stride, int64_t nv, int K) {
  const int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x;
  if (i >= nv) return;
  auto sv = ldc<VEC>(src + i * VEC);
  for (int k = 0; k < K; ++k) stv<VEC>(dst + (int64_t)k * stride + i * VEC, sv);
}

// bf16 operand copy of the weight matrices of replica blockIdx.y from its fp32 parameters.
__global__ __launch_bounds__(kThreads) void shadow_refresh_kernel(
    const float* __restrict__ x, uint16_t* __restrict__ shadow, ShadowMap map, int64_t stride,
    int64_t shadow_stride, int64_t nv) {
  const int k = blockIdx.y;
  const int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x;
  if (i >= nv) return;
  const int64_t so = shadow_offset4(map, i * 4);
  if (so < 0) return;
  store_bf16<4>(shadow + (int64_t)k * shadow_stride + so, ldc<4>(x + (int64_t)k * stride + i * 4));
}

// Row-major bf16 matrix of replica blockIdx.y -> blocked layout; one thread per 8 elements.
__global__ __launch_bounds__(kThreads) void rowmajor_to_b32s_kernel(
    const uint16_t* __restrict__ src, uint16_t* __restrict__ dst, int rows, int cols, int cblocks,
    int64_t dst_stride) {
  const int k = blockIdx.y;
  const int units = (cols + 7) / 8;
  const int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x;
  if (i >= (int64_t)rows * units) return;
  const int r = (int)(i / units), c = (int)(i % units) * 8;
  const uint16_t* sp = src + ((int64_t)k * rows + r) * cols + c;
  uint16_t* dp = dst + (int64_t)k * dst_stride + b32s_offset(r, c, cblocks);
  if (c + 8 <= cols && (cols % 8) == 0) {
    *reinterpret_cast<uint4*>(dp) = *reinterpret_cast<const uint4*>(sp);
  } else {
    for (int e = 0; e < 8 && c + e < cols; ++e) dp[e] = sp[e];
  }
}

__global__ __launch_bounds__(kThreads) void fill_zero_kernel(uint4* __restrict__ p, int64_t n16) {
  int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x;
  const int64_t step = (int64_t)gridDim.x * kThreads;
  for (; i < n16; i += step) p[i] = make_uint4(0, 0, 0, 0);
}

template <typename T>
__global__ __launch_bounds__(kThreads) void pad_rows_kernel(const T* __restrict__ s,
                                                           T* __restrict__ d, int64_t rows,
                                                           int cols, int ld) {
  const int64_t total = rows * cols;
  int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x;
  const int64_t step = (int64_t)gridDim.x * kThreads;
  for (; i < total; i += step) {
    const int64_t r = i / cols;
    const int c = (int)(i - r * cols);
    d[r * ld + c] = s[i];
  }
}

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15) == 0; }
inline unsigned blocks_for(int64_t n) { return (unsigned)((n + kThreads - 1) / kThreads); }
inline unsigned capped_blocks(int64_t n) {
  int64_t b = (n + kThreads - 1) / kThreads;
  return (unsigned)(b < 1 ? 1 : (b > 65536 ? 65536 : b));
}

}  // namespace

void launch_sumsq_partials(const float* g, int64_t g_stride, int64_t n, int K, double* partials,
                           int nblk, hipStream_t s) {
  dim3 grid(nblk, K);
  if (n % 4 == 0 && g_stride % 4 == 0 && aligned16(g)) {
    sumsq_partials_kernel<4><<<grid, kThreads, 0, s>>>(g, g_stride, n / 4, partials, nblk);
  } else {
    sumsq_partials_kernel<1><<<grid, kThreads, 0, s>>>(g, g_stride, n, partials, nblk);
  }
}

int launch_gram_dot(const float* G1, const float* G2, int64_t stride, int64_t n, int K, int pieces1,
                    int pieces2, int64_t piece_stride, double* partials, int64_t pstride, hipStream_t s) {
  // n and the strides are multiples of 4 (rows padded to 8 floats), the matrices 16-byte aligned
  const int64_t nv = n / 4;
  int64_t nb = (nv + 4 * kThreads - 1) / (4 * kThreads);
  const int nblk = (int)(nb < 1 ? 1 : (nb > 64 ? 64 : nb));
  gram_dot_partials_kernel<<<dim3(nblk, K), kThreads, 0, s>>>(G1, G2, stride, nv, pieces1, pieces2, piece_stride,
                                                              partials, pstride, nblk);
  return nblk;
}

void launch_norm_finish(const double* partials, int nblk, int64_t partials_stride, int K, float rho,
                        float gamma, float* norms, float* scale, const float* loss_rows, int B,
                        float* loss_out, hipStream_t s, int32_t* restart) {
  norm_finish_kernel<<<K, kThreads, 0, s>>>(partials, nblk, partials_stride, rho, gamma, norms,
                                            scale, loss_rows, B, loss_out, restart);
}

void launch_perturb(const float* x, const float* g, int64_t g_stride, const float* scale,
                    float* xt_f32, uint16_t* xt_bf16, const ShadowMap* map, int64_t shadow_stride,
                    int64_t stride, int64_t n, int K, hipStream_t s) {
  const bool vec = n % 4 == 0 && g_stride % 4 == 0 && stride % 4 == 0 && aligned16(g);
  ShadowMap none{};
  if (xt_bf16) {
    // bf16 mode only exists for the MLP layouts, which are always vector-aligned
    TileMap tm{};
    tm.n = map->n;
    int total = 0;
    for (int l = 0; l < map->n; ++l) {
      tm.first[l] = total;
      tm.ctiles[l] = (map->ldw[l] + 127) / 128;
      tm.rows[l] = (int)((map->end[l] - map->begin[l]) / map->ldw[l]);
      total += tm.ctiles[l] * ((tm.rows[l] + 7) / 8);
    }
    tm.first[map->n] = total;
    dim3 grid(total, K);
    perturb_tiled_kernel<<<grid, kThreads, 0, s>>>(x, g, g_stride, scale, xt_bf16, *map, tm,
                                                   shadow_stride, stride);
  } else if (vec) {
    dim3 grid(blocks_for(n / 4), K);
    if ((int64_t)K * n * 4 > kCacheResidentBytes)
      perturb_kernel<4, false, true><<<grid, kThreads, 0, s>>>(x, g, g_stride, scale, xt_f32, nullptr,
                                                               none, 0, stride, n / 4);
    else
      perturb_kernel<4, false, false><<<grid, kThreads, 0, s>>>(x, g, g_stride, scale, xt_f32,
                                                                nullptr, none, 0, stride, n / 4);
  } else {
    dim3 grid(blocks_for(n), K);
    perturb_kernel<1, false, true><<<grid, kThreads, 0, s>>>(x, g, g_stride, scale, xt_f32, nullptr,
                                                             none, 0, stride, n);
  }
}

template <typename NOISE>
void launch_descent_with(float* x, const float* g, int64_t g_stride, float* v, float* S,
                         const float* y, uint16_t* shadow, const ShadowMap* map,
                         int64_t shadow_stride, int64_t stride, int64_t n, int K,
                         const ReplicaScalars& lam, float lr, float mu, int nesterov,
                         const NOISE& noise, hipStream_t s, const int32_t* restart) {
  const bool vec = n % 4 == 0 && g_stride % 4 == 0 && stride % 4 == 0 && aligned16(g);
  ShadowMap none{};
  if (shadow) {
    const unsigned grid = blocks_for(n / 4) * (unsigned)K;
    descent_kernel<4, true, true, NOISE><<<grid, kThreads, 0, s>>>(
        x, g, g_stride, v, S, y, shadow, *map, shadow_stride, stride, n / 4, K, lam, lr, mu,
        nesterov, noise, restart);
  } else if (vec) {
    const unsigned grid = blocks_for(n / 4) * (unsigned)K;
    if ((int64_t)K * n * 4 > kCacheResidentBytes)
      descent_kernel<4, false, true, NOISE><<<grid, kThreads, 0, s>>>(
          x, g, g_stride, v, S, y, nullptr, none, 0, stride, n / 4, K, lam, lr, mu, nesterov, noise,
          restart);
    else
      descent_kernel<4, false, false, NOISE><<<grid, kThreads, 0, s>>>(
          x, g, g_stride, v, S, y, nullptr, none, 0, stride, n / 4, K, lam, lr, mu, nesterov, noise,
          restart);
  } else {
    const unsigned grid = blocks_for(n) * (unsigned)K;
    descent_kernel<1, false, true, NOISE><<<grid, kThreads, 0, s>>>(
        x, g, g_stride, v, S, y, nullptr, none, 0, stride, n, K, lam, lr, mu, nesterov, noise, restart);
  }
}

void launch_descent(float* x, const float* g, int64_t g_stride, float* v, float* S,
                    const float* y, uint16_t* shadow, const ShadowMap* map, int64_t shadow_stride,
                    int64_t stride, int64_t n, int K, const ReplicaScalars& lam, float lr, float mu,
                    int nesterov, const NoiseMap* noise, hipStream_t s, const int32_t* restart) {
  if (noise)
    launch_descent_with<NoiseMap>(x, g, g_stride, v, S, y, shadow, map, shadow_stride, stride, n, K,
                                  lam, lr, mu, nesterov, *noise, s, restart);
  else
    launch_descent_with<NoNoise>(x, g, g_stride, v, S, y, shadow, map, shadow_stride, stride, n, K,
                                 lam, lr, mu, nesterov, NoNoise{}, s, restart);
}

void launch_grad_mean(const float* src, int64_t src_stride, float* dst, int64_t dst_stride,
                      int64_t n, int K, int copies, hipStream_t s) {
  if (n % 4 == 0 && src_stride % 4 == 0 && dst_stride % 4 == 0 && aligned16(src) && aligned16(dst))
    grad_mean_kernel<4><<<blocks_for(n / 4), kThreads, 0, s>>>(src, src_stride, dst, dst_stride,
                                                               n / 4, K, copies);
  else
    grad_mean_kernel<1><<<blocks_for(n), kThreads, 0, s>>>(src, src_stride, dst, dst_stride, n, K,
                                                           copies);
}

void launch_center(float* S, float* y, float* gprev, int64_t stride, int64_t n,
                   const DueList& due, float inv_m, float beta, float lr_center, int has_prev,
                   hipStream_t s, int32_t* restart) {
  if (n % 4 == 0 && stride % 4 == 0) {
    center_kernel<4><<<blocks_for(n / 4), kThreads, 0, s>>>(S, y, gprev, stride, n / 4, due, inv_m,
                                                            beta, lr_center, has_prev, restart);
  } else {
    center_kernel<1><<<blocks_for(n), kThreads, 0, s>>>(S, y, gprev, stride, n, due, inv_m, beta,
                                                        lr_center, has_prev, restart);
  }
}

void launch_broadcast(const float* src, float* dst, int64_t stride, int64_t n, int K, hipStream_t s) {
  // internal buffers only: n and stride are multiples of 4 by construction
  broadcast_kernel<4><<<blocks_for(n / 4), kThreads, 0, s>>>(src, dst, stride, n / 4, K);
}

void launch_shadow_refresh(const float* x, uint16_t* shadow, const ShadowMap& map, int64_t stride,
                           int64_t shadow_stride, int64_t n, int K, hipStream_t s) {
  dim3 grid(blocks_for(n / 4), K);
  shadow_refresh_kernel<<<grid, kThreads, 0, s>>>(x, shadow, map, stride, shadow_stride, n / 4);
}

void launch_rowmajor_to_b32s(const uint16_t* src, uint16_t* dst, int rows, int cols, int K,
                             hipStream_t s) {
  const int64_t work = (int64_t)rows * ((cols + 7) / 8);
  dim3 grid(blocks_for(work), K);
  rowmajor_to_b32s_kernel<<<grid, kThreads, 0, s>>>(src, dst, rows, cols, b32s_blocks(cols),
                                                    b32s_size(rows, cols));
}

void launch_fill_zero(void* p, size_t bytes, hipStream_t s) {
  if (bytes == 0) return;
  fill_zero_kernel<<<capped_blocks((int64_t)(bytes / 16)), kThreads, 0, s>>>(
      reinterpret_cast<uint4*>(p), (int64_t)(bytes / 16));
}

void launch_pad_rows(const void* src, void* dst, int64_t rows, int cols, int ld_dst, int elem,
                     hipStream_t s) {
  const unsigned grid = capped_blocks(rows * cols);
  if (elem == 4)
    pad_rows_kernel<float><<<grid, kThreads, 0, s>>>((const float*)src, (float*)dst, rows, cols,
                                                     ld_dst);
  else
    pad_rows_kernel<uint16_t><<<grid, kThreads, 0, s>>>((const uint16_t*)src, (uint16_t*)dst, rows,
                                                        cols, ld_dst);
}

}  // namespace lsam
