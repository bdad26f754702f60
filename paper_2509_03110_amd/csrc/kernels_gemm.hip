// K-batched replica GEMMs on the MFMA units: forward (Z = A W^T + b), input gradient
// (dA = dZ W, masked by ReLU') and weight gradient (dW = dZ^T A), for fp32 operands
// (v_mfma_f32_32x32x2_f32) and bf16 operands (v_mfma_f32_32x32x16_bf16), fp32 accumulate.
//
// One formulation covers all three:  C[m,n] = sum_k A(m,k) * B(n,k).
// An operand is k-major if k is its contiguous index in memory, m-major otherwise.  Either
// way it is staged through LDS in "units" of 16 bytes holding UE consecutive k of one row
// (UE = 4 floats or 8 bf16).  k-major operands are loaded as units straight from memory;
// m-major operands are loaded as UE rows x 16 bytes per thread and transposed in registers
// (free for fp32, a few byte-permutes for bf16), so that the MFMA feed is the same 128-bit
// LDS read in every case.  A workgroup is 4 wavefronts in a 2x2 arrangement; each wavefront
// owns a (BM/2)x(BN/2) block of 32x32 MFMA tiles.
#include "engine.h"

namespace lsam {
namespace {

constexpr int kThreads = 256;
constexpr int BKU = 8;   // 16-byte units per row per k-step: 128 bytes of k per step

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned short u16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

struct GemmParams {
  const char* A; long long strideA; int ldA;
  const char* B; long long strideB; int ldB;
  char* C; long long strideC; int ldC;
  int M, N, Kd, batch;
  int tilesM, tilesN, total, chunks;
  int epilogue;
  const float* bias; long long strideBias;
  const float* bias_dir; const float* bias_scale;
  const char* mask; long long strideMask; int ldMask;
};

template <typename T> struct Op;
template <> struct Op<float> { static constexpr int UE = 4; };
template <> struct Op<__bf16> { static constexpr int UE = 8; };

// Row position inside an LDS tile: rows are permuted inside groups of UE so that both the
// transposing writes (lanes UE rows apart) and the MFMA reads (lanes on consecutive rows)
// spread over the banks.
template <int UE>
__device__ __forceinline__ int swz(int r) { return r ^ ((r / UE) & (UE - 1)); }

// Loads one operand tile (R rows x BKU units) from global memory into registers.
template <typename T, int R, bool KMAJOR>
struct TileLoader {
  static constexpr int UE = Op<T>::UE;
  static constexpr int NUNITS = KMAJOR ? (R * BKU / kThreads) : 0;                 // per thread
  static constexpr int NBLK_TOTAL = BKU * (R / UE);
  static constexpr int NBLK = KMAJOR ? 0 : (NBLK_TOTAL + kThreads - 1) / kThreads;  // per thread
  static constexpr int NREG = KMAJOR ? (NUNITS > 0 ? NUNITS : 1) : NBLK * UE;
  u32x4 reg[NREG];

  // base: operand of this replica; row0: first tile row; k0u: first k-unit of this step;
  // rows: row extent with readable padding up to a multiple of UE; kd: true k extent.
  __device__ __forceinline__ void load(const T* __restrict__ base, int ld, int row0, int rows,
                                       int k0u, int kd, int tid) {
    const u32x4 zero = {0u, 0u, 0u, 0u};
    if constexpr (KMAJOR) {
      const int kunits = (kd + UE - 1) / UE;
#pragma unroll
      for (int j = 0; j < NUNITS; ++j) {
        const int u = tid + kThreads * j;
        const int r = row0 + u / BKU, ku = k0u + u % BKU;
        reg[j] = (r < rows && ku < kunits)
                     ? *reinterpret_cast<const u32x4*>(base + (long long)r * ld + ku * UE)
                     : zero;
      }
    } else {
      const int rows_up = (rows + UE - 1) / UE * UE;
#pragma unroll
      for (int j = 0; j < NBLK; ++j) {
        const int b = tid + kThreads * j;
        const int mg = b % (R / UE), kb = b / (R / UE);
        const int m = row0 + mg * UE;
#pragma unroll
        for (int i = 0; i < UE; ++i) {
          const int k = (k0u + kb) * UE + i;
          reg[j * UE + i] = (b < NBLK_TOTAL && m < rows_up && k < kd)
                                ? *reinterpret_cast<const u32x4*>(base + (long long)k * ld + m)
                                : zero;
        }
      }
    }
  }

  // Writes the registers to the LDS tile laid out as units [BKU][R + 1].
  __device__ __forceinline__ void store(u32x4* __restrict__ lds, int tid) const {
    if constexpr (KMAJOR) {
#pragma unroll
      for (int j = 0; j < NUNITS; ++j) {
        const int u = tid + kThreads * j;
        lds[(u % BKU) * (R + 1) + swz<UE>(u / BKU)] = reg[j];
      }
    } else {
#pragma unroll
      for (int j = 0; j < NBLK; ++j) {
        const int b = tid + kThreads * j;
        if (b < NBLK_TOTAL) {
          const int mg = b % (R / UE), kb = b / (R / UE);
#pragma unroll
          for (int e = 0; e < UE; ++e) {
            u32x4 unit;
            if constexpr (UE == 4) {
              unit[0] = reg[j * 4 + 0][e];
              unit[1] = reg[j * 4 + 1][e];
              unit[2] = reg[j * 4 + 2][e];
              unit[3] = reg[j * 4 + 3][e];
            } else {
#pragma unroll
              for (int q = 0; q < 4; ++q) {
                const unsigned lo = reg[j * 8 + 2 * q][e / 2];
                const unsigned hi = reg[j * 8 + 2 * q + 1][e / 2];
                unit[q] = (e & 1) ? ((lo >> 16) | (hi & 0xFFFF0000u))
                                  : ((lo & 0xFFFFu) | (hi << 16));
              }
            }
            lds[kb * (R + 1) + swz<UE>(mg * UE + e)] = unit;
          }
        }
      }
    }
  }
};

__device__ __forceinline__ float widen(float v) { return v; }
__device__ __forceinline__ float widen(__bf16 v) { return static_cast<float>(v); }

template <typename T, typename TC, int BM, int BN, bool A_KMAJOR, bool B_KMAJOR>
__global__ __launch_bounds__(kThreads) void gemm_kernel(GemmParams p) {
  constexpr int UE = Op<T>::UE;
  constexpr int TM = BM / 64, TN = BN / 64;
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  u32x4* ldsA = reinterpret_cast<u32x4*>(smem);
  u32x4* ldsB = ldsA + BKU * (BM + 1);

  // Workgroup -> tile.  Hardware deals consecutive workgroup ids round-robin over the 8
  // XCDs; remap so that each XCD walks a contiguous range of tiles (tiles that share a
  // weight panel then share one L2).
  const int w = blockIdx.x;
  const int logical = (w % 8) * p.chunks + w / 8;
  if (logical >= p.total) return;
  const int tm_idx = logical % p.tilesM;
  const int tn_idx = (logical / p.tilesM) % p.tilesN;
  const int bat = logical / (p.tilesM * p.tilesN);
  const int m0 = tm_idx * BM, n0 = tn_idx * BN;

  const T* A = reinterpret_cast<const T*>(p.A) + (long long)bat * p.strideA;
  const T* B = reinterpret_cast<const T*>(p.B) + (long long)bat * p.strideB;

  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  const int wm0 = (wave >> 1) * (BM / 2), wn0 = (wave & 1) * (BN / 2);
  const int l32 = lane & 31, h = lane >> 5;

  f32x16 acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

  TileLoader<T, BM, A_KMAJOR> la;
  TileLoader<T, BN, B_KMAJOR> lb;
  const int ksteps = (p.Kd + BKU * UE - 1) / (BKU * UE);
  la.load(A, p.ldA, m0, p.M, 0, p.Kd, tid);
  lb.load(B, p.ldB, n0, p.N, 0, p.Kd, tid);

  for (int ks = 0; ks < ksteps; ++ks) {
    la.store(ldsA, tid);
    lb.store(ldsB, tid);
    __syncthreads();
    if (ks + 1 < ksteps) {
      la.load(A, p.ldA, m0, p.M, (ks + 1) * BKU, p.Kd, tid);
      lb.load(B, p.ldB, n0, p.N, (ks + 1) * BKU, p.Kd, tid);
    }
#pragma unroll
    for (int kc = 0; kc < BKU / 2; ++kc) {
      const int ku = kc * 2 + h;
      u32x4 fa[TM], fb[TN];
#pragma unroll
      for (int i = 0; i < TM; ++i) fa[i] = ldsA[ku * (BM + 1) + swz<UE>(wm0 + i * 32 + l32)];
#pragma unroll
      for (int j = 0; j < TN; ++j) fb[j] = ldsB[ku * (BN + 1) + swz<UE>(wn0 + j * 32 + l32)];
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) {
          if constexpr (UE == 4) {
            const f32x4 a = __builtin_bit_cast(f32x4, fa[i]);
            const f32x4 b = __builtin_bit_cast(f32x4, fb[j]);
#pragma unroll
            for (int e = 0; e < 4; ++e)
              acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[e], b[e], acc[i][j], 0, 0, 0);
          } else {
            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
                __builtin_bit_cast(bf16x8, fa[i]), __builtin_bit_cast(bf16x8, fb[j]), acc[i][j], 0,
                0, 0);
          }
        }
    }
    __syncthreads();
  }

  // Epilogue.  Accumulator element e of a 32x32 tile: row (e/4)*8 + h*4 + e%4, column l32.
  TC* C = reinterpret_cast<TC*>(p.C) + (long long)bat * p.strideC;
  const float* bias = p.bias ? p.bias + (long long)bat * p.strideBias : nullptr;
  const float* bias_dir = p.bias_dir ? p.bias_dir + (long long)bat * p.strideBias : nullptr;
  const float bias_sc = p.bias_dir ? p.bias_scale[bat] : 0.f;
  const T* mask = p.mask ? reinterpret_cast<const T*>(p.mask) + (long long)bat * p.strideMask
                         : nullptr;
#pragma unroll
  for (int j = 0; j < TN; ++j) {
    const int n = n0 + wn0 + j * 32 + l32;
    if (n >= p.N) continue;
    float bv = 0.f;
    if (p.epilogue == EPI_BIAS || p.epilogue == EPI_BIAS_RELU) {
      bv = bias[n];
      if (bias_dir) bv = bv + bias_sc * bias_dir[n];   // bias of the perturbed point
    }
#pragma unroll
    for (int i = 0; i < TM; ++i) {
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        const int m = m0 + wm0 + i * 32 + (e / 4) * 8 + h * 4 + (e % 4);
        if (m >= p.M) continue;
        float v = acc[i][j][e] + bv;
        if (p.epilogue == EPI_BIAS_RELU) v = v > 0.f ? v : 0.f;
        if (p.epilogue == EPI_MASK) {
          if (!(widen(mask[(long long)m * p.ldMask + n]) > 0.f)) v = 0.f;
        }
        C[(long long)m * p.ldC + n] = static_cast<TC>(v);
      }
    }
  }
}

template <typename T, typename TC, int BM, int BN, bool AK, bool BK_>
int launch_one(const GemmParams& p0, hipStream_t s) {
  GemmParams p = p0;
  p.tilesM = (p.M + BM - 1) / BM;
  p.tilesN = (p.N + BN - 1) / BN;
  p.total = p.tilesM * p.tilesN * p.batch;
  p.chunks = (p.total + 7) / 8;
  const size_t smem = (size_t)BKU * ((BM + 1) + (BN + 1)) * 16;
  auto kern = gemm_kernel<T, TC, BM, BN, AK, BK_>;
  static bool attr_set = false;   // per instantiation
  if (!attr_set) {
    if (hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                            hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem) != hipSuccess)
      return -1;
    attr_set = true;
  }
  kern<<<p.chunks * 8, kThreads, smem, s>>>(p);
  return 0;
}

template <typename T, typename TC, bool AK, bool BK_>
int launch_tiled(const GemmParams& p, hipStream_t s) {
  // Largest tile that still yields at least ~2 workgroups per compute unit.
  auto tiles = [&](int bm, int bn) {
    return (long long)((p.M + bm - 1) / bm) * ((p.N + bn - 1) / bn) * p.batch;
  };
  if (p.M >= 256 && p.N >= 256 && tiles(256, 256) >= 512)
    return launch_one<T, TC, 256, 256, AK, BK_>(p, s);
  if (p.M >= 128 && p.N >= 128 && tiles(128, 128) >= 512)
    return launch_one<T, TC, 128, 128, AK, BK_>(p, s);
  return launch_one<T, TC, 64, 64, AK, BK_>(p, s);
}

template <typename T, typename TC>
int launch_layout(const GemmDesc& d, const GemmParams& p, hipStream_t s) {
  if (d.a_kmajor && d.b_kmajor) return launch_tiled<T, TC, true, true>(p, s);
  if (d.a_kmajor && !d.b_kmajor) return launch_tiled<T, TC, true, false>(p, s);
  if (!d.a_kmajor && !d.b_kmajor) return launch_tiled<T, TC, false, false>(p, s);
  return -1;
}

}  // namespace

int launch_gemm(const GemmDesc& d, hipStream_t s) {
  GemmParams p;
  p.A = (const char*)d.A; p.strideA = d.strideA; p.ldA = d.ldA;
  p.B = (const char*)d.B; p.strideB = d.strideB; p.ldB = d.ldB;
  p.C = (char*)d.C; p.strideC = d.strideC; p.ldC = d.ldC;
  p.M = d.M; p.N = d.N; p.Kd = d.Kd; p.batch = d.batch;
  p.tilesM = p.tilesN = p.total = p.chunks = 0;
  p.epilogue = d.epilogue;
  p.bias = d.bias; p.strideBias = d.strideBias;
  p.bias_dir = d.bias_dir; p.bias_scale = d.bias_scale;
  p.mask = (const char*)d.mask; p.strideMask = d.strideMask; p.ldMask = d.ldMask;
  if (d.M <= 0 || d.N <= 0 || d.Kd <= 0 || d.batch <= 0) return -1;
  // 16-byte units: pitches must be multiples of 8 elements and bases 16-byte aligned.
  if ((d.ldA % 8) || (d.ldB % 8) || ((uintptr_t)d.A & 15) || ((uintptr_t)d.B & 15)) return -1;
  if (d.in_bf16) {
    if ((d.strideA % 8) || (d.strideB % 8)) return -1;
    if (d.out_bf16) return launch_layout<__bf16, __bf16>(d, p, s);
    return launch_layout<__bf16, float>(d, p, s);
  }
  if ((d.strideA % 4) || (d.strideB % 4)) return -1;
  if (d.out_bf16) return -1;
  return launch_layout<float, float>(d, p, s);
}

}  // namespace lsam
