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
// LDS read in every case.  Global loads are buffer loads: rows past the end of an operand
// come back as zeros from the hardware range check instead of through branches.
//
// A workgroup is 4 wavefronts in a 2x2 arrangement; each wavefront owns a (BM/2)x(BN/2)
// block of 32x32 MFMA tiles.  LDS is double buffered (one barrier per k-step): the next
// k-step's global loads are issued before the MFMAs of the current one and written to the
// other LDS buffer after them; operand fragments are double buffered in registers so LDS
// reads of the next 16 (bf16) / 8 (fp32) k overlap the MFMAs of the current ones.
// The MFMA is issued with the roles swapped (rows <- B operand, columns <- A operand), so
// that a lane ends up with 4 consecutive n of one row m: 16-byte stores in the epilogue.
#include <atomic>
#include <type_traits>

#include "engine.h"

namespace lsam {
namespace {

constexpr int kThreads = 256;

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

// An operand that is the unfolded image of a 3x3 convolution (stride 1, zero rim 1) without
// the unfolded image being stored: element (pixel, tap * C + c) is image[pixel shifted by the
// tap][c], zero outside the image.  Pixels are rows of [B][H][W][C]; 1/W and 1/H serve the
// pixel -> (row, column) decode (exact for pixel indices below 2^24).
struct ConvMap {
  int C, H, W;
  float invW, invH;
  int step_rows;   // image rows a k-step of 32 pixels advances, if 4 | W and W | 32; else 0
};

struct GemmParams {
  ConvMap cm;
  const char* A; long long strideA; int ldA;
  const char* B; long long strideB; int ldB;
  char* C; long long strideC; int ldC;
  int M, N, Kd, batch;
  int tilesM, tilesN, total, chunks;
  int epilogue;
  const float* bias; long long strideBias;
  const float* bias_dir; const float* bias_scale;
  const char* mask; long long strideMask; int ldMask;
  // split-K: the contraction is cut into `splits` ranges of `steps_per_split` k-steps, each
  // range owned by its own workgroup, which writes raw fp32 sums to partial[split]
  float* partial; long long strideSplit; int ldP;
  int splits, steps_per_split;
  // optional sum of squares of the stored results, one slot per workgroup that stores them
  double* sumsq; long long strideSumsq;
};

// Sum over a 256-thread workgroup in a fixed order (lanes by xor-shuffle, then the four
// wavefronts in turn); the result is valid in thread 0.
__device__ __forceinline__ double workgroup_sum(double v) {
  __shared__ double part[4];
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
  if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = v;
  __syncthreads();
  return threadIdx.x == 0 ? (part[0] + part[1]) + (part[2] + part[3]) : 0.0;
}

template <typename T> struct Op;
template <> struct Op<float> { static constexpr int UE = 4; };
template <> struct Op<__bf16> { static constexpr int UE = 8; };

constexpr unsigned kOob = 0x7FFFFFF0u;   // byte offset past any operand: load returns zeros

// Row position inside an LDS tile: rows are permuted inside aligned groups of UE.  A 128-bit
// LDS access is served 8 lanes (128 bytes = all banks) at a time.  The MFMA reads put 8 lanes
// on 8 consecutive rows, which any permutation inside groups of UE keeps on 8 distinct
// 16-byte slots.  The transposing writes of an m-major operand put lane i on row UE*i + e, so
// 8 consecutive lanes hit slots UE*(i mod 2) + (e permuted) modulo 8: the permutation must
// differ for lanes two apart, hence bits of r / (2 UE).  (Taken from r / UE, lanes i and
// i + 2 collided: 26 % of the LDS cycles of the fp32 weight-gradient GEMM were bank
// conflicts; now none.)
template <int UE>
__device__ __forceinline__ int swz(int r) { return r ^ ((r / (2 * UE)) & (UE - 1)); }
// The same for tiles of 8-byte units (fp32 operands rounded to bfloat16 on their way into LDS).
// A 64-bit LDS access is served 16 lanes at a time.  The MFMA reads put 16 lanes on 16
// consecutive rows: 128 contiguous bytes under any permutation inside groups of four.  The
// transposing writes put lane i on row 4 i + e, 32 bytes apart, so lanes four apart meet on the
// same banks unless their permutations differ: bits of r / 16.  The k-major writes put 8 lanes
// on the 8 k-units of a row and the next 8 on the next row; with a k-unit pitch of R + 2 units
// (2 mod 16) the first 8 take the even 8-byte slots and the second 8 the odd ones.
__device__ __forceinline__ int swz_half(int r) { return r ^ ((r / 16) & 3); }

// Loads one operand tile (R rows x BKU units of 16 bytes: 16*BKU bytes of k per k-step) from
// global memory into registers and writes it to LDS laid out as units [BKU][R + 1].
__device__ __forceinline__ void pixel_coords(int k, const ConvMap& cm, int& i, int& j) {
  int q = (int)((float)k * cm.invW);
  int r = k - q * cm.W;
  if (r < 0) { r += cm.W; --q; } else if (r >= cm.W) { r -= cm.W; ++q; }
  j = r;
  const int q2 = (int)((float)q * cm.invH);
  int r2 = q - q2 * cm.H;
  if (r2 < 0) r2 += cm.H; else if (r2 >= cm.H) r2 -= cm.H;
  i = r2;
}

// IMPL: 0 = the operand is stored as described by (ld, rows); 1 = k-major operand that is an
// unfolded image (rows = pixels, k = tap * C + c; C a multiple of the k-step so that a k-step
// lies inside one tap); 2 = m-major operand that is an unfolded image (k = pixels, columns =
// tap * C + c).
template <typename T, int R, bool KMAJOR, int BKU, int IMPL = 0>
struct TileLoader {
  static constexpr int UE = Op<T>::UE;
  static constexpr int ES = sizeof(T);
  static constexpr int NUNITS = KMAJOR ? (R * BKU / kThreads) : 0;                 // per thread
  static constexpr int NBLK_TOTAL = BKU * (R / UE);
  static constexpr int NBLK = KMAJOR ? 0 : (NBLK_TOTAL + kThreads - 1) / kThreads;  // per thread
  static constexpr int NREG = KMAJOR ? (NUNITS > 0 ? NUNITS : 1) : NBLK * UE;
  static constexpr int NSTORE = NREG;   // 16-byte LDS writes per thread and k-step
  u32x4 reg[NREG];
  static constexpr int NPRE = IMPL == 1 ? NUNITS : (IMPL == 2 ? NBLK : 1);
  int pre_off[IMPL ? NPRE : 1];   // byte offset that does not change from k-step to k-step
  int pre_i[IMPL ? NPRE : 1];     // IMPL 1: image row of the unit's pixel; 2: row shift of its tap
  int pre_j[IMPL ? NPRE : 1];     // IMPL 1: image column;                 2: column shift
  // IMPL 2: image row and column of each block's first pixel, carried from one k-step to the
  // next (k-steps come in order: 32 pixels further the column is the same when W | 32 and the
  // row has advanced by 32 / W), so that only the first k-step pays for a decode
  int cur_i[IMPL == 2 ? NPRE : 1], cur_j[IMPL == 2 ? NPRE : 1];
  int next_k0u = -1;

  // What stays fixed while a tile is computed.  row0/rows: first tile row and row extent
  // (IMPL 1: pixels; IMPL 2: columns tap * C + c, extent 9 C).
  __device__ __forceinline__ void prepare(const ConvMap& cm, int row0, int rows, int tid) {
    static_assert(IMPL == 0 || UE == 4, "implicit unfolding is built for fp32 operands");
    if constexpr (IMPL == 1) {
#pragma unroll
      for (int j = 0; j < NUNITS; ++j) {
        const int u = tid + kThreads * j;
        const int r = row0 + u / BKU;
        if (r < rows) {
          pixel_coords(r, cm, pre_i[j], pre_j[j]);
          pre_off[j] = (r * cm.C + (u % BKU) * UE) * ES;
        } else {
          pre_i[j] = pre_j[j] = 1 << 20;   // fails every bounds test
          pre_off[j] = 0;
        }
      }
    } else if constexpr (IMPL == 2) {
#pragma unroll
      for (int j = 0; j < NBLK; ++j) {
        const int b = tid + kThreads * j;
        const int m = row0 + (b % (R / UE)) * UE;
        if (b < NBLK_TOTAL && m < rows) {
          const int tap = m / cm.C, c = m - tap * cm.C;
          pre_i[j] = tap / 3 - 1;
          pre_j[j] = tap % 3 - 1;
          pre_off[j] = ((pre_i[j] * cm.W + pre_j[j]) * cm.C + c) * ES;
        } else {
          pre_i[j] = pre_j[j] = 1 << 20;
          pre_off[j] = 0;
        }
      }
    }
  }

  // k0u: first k-unit of this step; kd: true k extent (IMPL 1: 9 C; IMPL 2: pixels).
  __device__ __forceinline__ void load_unfolded(__amdgpu_buffer_rsrc_t rsrc, const ConvMap& cm, int k0u,
                                                int kd, int tid) {
    if constexpr (IMPL == 1) {
      const int e0 = k0u * UE;
      const int tap = e0 / cm.C, c0 = e0 - tap * cm.C;
      const int du = tap / 3 - 1, dv = tap % 3 - 1;
      const int shift = ((du * cm.W + dv) * cm.C + c0) * ES;
#pragma unroll
      for (int j = 0; j < NUNITS; ++j) {
        const bool ok = e0 < kd && (unsigned)(pre_i[j] + du) < (unsigned)cm.H &&
                        (unsigned)(pre_j[j] + dv) < (unsigned)cm.W;
        reg[j] = __builtin_amdgcn_raw_buffer_load_b128(rsrc, ok ? (unsigned)(pre_off[j] + shift) : kOob,
                                                       0, 0);
      }
    } else if constexpr (IMPL == 2) {
#pragma unroll
      for (int j = 0; j < NBLK; ++j) {
        const int b = tid + kThreads * j;
        const int kb = b / (R / UE);
        // the block's four pixels start at a multiple of 4: with 4 | W they share an image row
        // and one decode serves them all
        const bool one_row = (cm.W & 3) == 0;
        int pi0 = 0, pj0 = 0;
        if (BKU * UE == 32 && cm.step_rows > 0 && k0u == next_k0u) {
          pi0 = cur_i[j];
          pj0 = cur_j[j];
        } else if (one_row) {
          pixel_coords((k0u + kb) * UE, cm, pi0, pj0);
        }
        if (BKU * UE == 32 && cm.step_rows > 0) {
          int ni = pi0 + cm.step_rows;
          while (ni >= cm.H) ni -= cm.H;
          cur_i[j] = ni;
          cur_j[j] = pj0;
        }
#pragma unroll
        for (int i = 0; i < UE; ++i) {
          const int k = (k0u + kb) * UE + i;
          int pi = pi0, pj = pj0 + i;
          if (!one_row) pixel_coords(k, cm, pi, pj);
          const bool ok = k < kd && (unsigned)(pi + pre_i[j]) < (unsigned)cm.H &&
                          (unsigned)(pj + pre_j[j]) < (unsigned)cm.W;
          reg[j * UE + i] = __builtin_amdgcn_raw_buffer_load_b128(
              rsrc, ok ? (unsigned)(k * cm.C * ES + pre_off[j]) : kOob, 0, 0);
        }
      }
      next_k0u = k0u + BKU;
    }
  }

  // rsrc covers the operand of this replica: rows*ld elements (k-major) or kd*ld (m-major),
  // so a row index past the end is out of range by construction.  row0: first tile row;
  // k0u: first k-unit of this step; rows: row extent; kd: true k extent.
  __device__ __forceinline__ void load(__amdgpu_buffer_rsrc_t rsrc, int ld, int row0, int rows,
                                       int k0u, int kd, int tid) {
    if constexpr (KMAJOR) {
      const int kunits = (kd + UE - 1) / UE;
#pragma unroll
      for (int j = 0; j < NUNITS; ++j) {
        const int u = tid + kThreads * j;
        const int r = row0 + u / BKU, ku = k0u + u % BKU;
        const unsigned off = (unsigned)(r * ld + ku * UE) * ES;
        reg[j] = __builtin_amdgcn_raw_buffer_load_b128(rsrc, (r < rows && ku < kunits) ? off : kOob,
                                                       0, 0);
      }
    } else {
      // Rows k >= kd lie past the end of the buffer and read as zeros by themselves; a
      // column group past the operand's width is sent there through its column offset.
      const int rows_up = (rows + UE - 1) / UE * UE;
#pragma unroll
      for (int j = 0; j < NBLK; ++j) {
        const int b = tid + kThreads * j;
        const int mg = b % (R / UE), kb = b / (R / UE);
        const int m = row0 + mg * UE;
        const unsigned moff = (b < NBLK_TOTAL && m < rows_up) ? (unsigned)m * ES : kOob;
#pragma unroll
        for (int i = 0; i < UE; ++i) {
          const int k = (k0u + kb) * UE + i;
          const unsigned koff = (k < kd) ? (unsigned)(k * ld) * ES : 0u;
          reg[j * UE + i] = __builtin_amdgcn_raw_buffer_load_b128(
              rsrc, (k < kd) ? koff + moff : kOob, 0, 0);
        }
      }
    }
  }

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
        if (NBLK_TOTAL % kThreads == 0 || b < NBLK_TOTAL) {
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
                // bytes of {hi,lo}: keep the even (low) or the odd (high) halfwords
                unit[q] = (e & 1) ? __builtin_amdgcn_perm(hi, lo, 0x07060302u)
                                  : __builtin_amdgcn_perm(hi, lo, 0x05040100u);
              }
            }
            lds[kb * (R + 1) + swz<UE>(mg * UE + e)] = unit;
          }
        }
      }
    }
  }

  // The same tile (fp32 in registers) written as bfloat16: units of 8 bytes, four k each, at the
  // same unit positions.  For the arithmetic mode that rounds fp32 operands on their way into
  // the matrix unit: rounding here instead of after the LDS read halves the LDS traffic.
  __device__ __forceinline__ void store(u32x2* __restrict__ lds, int tid) const {
    static_assert(UE == 4, "fp32 operands");
    if constexpr (KMAJOR) {
#pragma unroll
      for (int j = 0; j < NUNITS; ++j) {
        const int u = tid + kThreads * j;
        lds[(u % BKU) * (R + 2) + swz_half(u / BKU)] = round4(__builtin_bit_cast(f32x4, reg[j]));
      }
    } else {
#pragma unroll
      for (int j = 0; j < NBLK; ++j) {
        const int b = tid + kThreads * j;
        if (NBLK_TOTAL % kThreads == 0 || b < NBLK_TOTAL) {
          const int mg = b % (R / UE), kb = b / (R / UE);
          // round each loaded row (one k, four m), then transpose the 4x4 block of halfwords
          u32x2 c[4];
#pragma unroll
          for (int q = 0; q < 4; ++q) c[q] = round4(__builtin_bit_cast(f32x4, reg[j * 4 + q]));
#pragma unroll
          for (int e = 0; e < UE; ++e) {
            const unsigned sel = (e & 1) ? 0x07060302u : 0x05040100u;   // odd / even halfwords of {hi, lo}
            u32x2 unit;
            unit[0] = __builtin_amdgcn_perm(c[1][e / 2], c[0][e / 2], sel);
            unit[1] = __builtin_amdgcn_perm(c[3][e / 2], c[2][e / 2], sel);
            lds[kb * (R + 2) + swz_half(mg * UE + e)] = unit;
          }
        }
      }
    }
  }
  static __device__ __forceinline__ u32x2 round4(const f32x4& v) {
    typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
    const bf16x2 lo = {static_cast<__bf16>(v[0]), static_cast<__bf16>(v[1])};
    const bf16x2 hi = {static_cast<__bf16>(v[2]), static_cast<__bf16>(v[3])};
    return u32x2{__builtin_bit_cast(unsigned, lo), __builtin_bit_cast(unsigned, hi)};
  }
};

template <typename T> struct Pack;
template <> struct Pack<float> {
  typedef f32x4 vec;
  static __device__ __forceinline__ vec from(const f32x4& v) { return v; }
  static __device__ __forceinline__ float one(float v) { return v; }
};
template <> struct Pack<__bf16> {
  typedef u32x2 vec;
  static __device__ __forceinline__ vec from(const f32x4& v) {
    typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
    bf16x2 lo = {static_cast<__bf16>(v[0]), static_cast<__bf16>(v[1])};
    bf16x2 hi = {static_cast<__bf16>(v[2]), static_cast<__bf16>(v[3])};
    vec o;
    o[0] = __builtin_bit_cast(unsigned, lo);
    o[1] = __builtin_bit_cast(unsigned, hi);
    return o;
  }
  static __device__ __forceinline__ __bf16 one(float v) { return static_cast<__bf16>(v); }
};

// Buffer resource for one replica's operand.  Base and size are the same for every lane;
// passing them through readfirstlane tells the compiler so (the descriptor must sit in
// scalar registers, and a descriptor it believes to vary per lane costs a loop per load).
template <typename T>
__device__ __forceinline__ __amdgpu_buffer_rsrc_t make_rsrc(const T* base, unsigned bytes) {
  const unsigned long long a = reinterpret_cast<unsigned long long>(base);
  const unsigned lo = __builtin_amdgcn_readfirstlane((unsigned)a);
  const unsigned hi = __builtin_amdgcn_readfirstlane((unsigned)(a >> 32));
  void* ptr = reinterpret_cast<void*>(((unsigned long long)hi << 32) | lo);
  return __builtin_amdgcn_make_buffer_rsrc(ptr, 0, __builtin_amdgcn_readfirstlane(bytes),
                                           0x00020000);
}

// Scheduling hints (sched_group_barrier): spread N instructions of class MASK evenly over M
// MFMAs, in that order.  Classes: 0x008 MFMA, 0x020 VMEM read, 0x100 LDS read, 0x200 LDS write.
template <int MASK, int N, int M, int I>
struct Interleave {
  static __device__ __forceinline__ void run() {
    constexpr int ops = N * (I + 1) / M - N * I / M;
    if constexpr (ops > 0) __builtin_amdgcn_sched_group_barrier(MASK, ops, 0);
    __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
    if constexpr (I + 1 < M) Interleave<MASK, N, M, I + 1>::run();
  }
};
// One k-chunk: ND fragment reads, then NX other memory instructions (class XMASK), laid over
// the chunk's NM MFMAs.
template <int ND, int NX, int XMASK, int NM>
struct Pipeline {
  static __device__ __forceinline__ void run() {
    constexpr int MA = NX > 0 ? (NM + 1) / 2 : NM;
    constexpr int MB = NM - MA;
    Interleave<0x100, ND, MA, 0>::run();
    if constexpr (MB > 0) Interleave<XMASK, NX, MB, 0>::run();
  }
};

__device__ __forceinline__ float widen(float v) { return v; }
__device__ __forceinline__ float widen(__bf16 v) { return static_cast<float>(v); }

// CONV: 0 = both operands stored; 1 = A is an unfolded image (k-major); 2 = B is one (m-major).
// BF16MATH (fp32 operands only): the operands stay fp32 in memory; they are rounded to bfloat16
// (round to nearest even) as the loaded tile is written to LDS, in units of 8 instead of 16
// bytes, and each pair of k-chunks feeds one v_mfma_f32_32x32x16_bf16 instead of eight
// v_mfma_f32_32x32x2_f32 -- the rounding rule of the bf16 configurations (only what enters the
// matrix unit is rounded) at fp32 memory traffic and half the LDS traffic.
// Which k a lane's eight values stand for does not matter as long as both operands agree: a
// lane takes the four of its unit in the even chunk and the four of its unit in the odd one.
template <typename T, typename TC, int BM, int BN, int BKU, bool A_KMAJOR, bool B_KMAJOR, int OCC,
          int CONV = 0, bool BF16MATH = false>
__global__ __launch_bounds__(kThreads, OCC) void gemm_kernel(GemmParams p) {
  static_assert(!BF16MATH || Op<T>::UE == 4, "bf16 math is a mode of the fp32-operand kernel");
  static_assert(CONV == 0 || (CONV == 1 && A_KMAJOR) || (CONV == 2 && !B_KMAJOR), "operand layout");
  constexpr int UE = Op<T>::UE;
  constexpr int TM = BM / 64, TN = BN / 64;
  constexpr int PAD = BF16MATH ? 2 : 1;          // k-unit pitch of a tile is its rows + PAD units
  constexpr int A_UNITS = BKU * (BM + PAD), B_UNITS = BKU * (BN + PAD);
  constexpr int STAGE_UNITS = A_UNITS + B_UNITS;
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  typedef typename std::conditional<BF16MATH, u32x2, u32x4>::type unit_t;   // one LDS unit: 4 k of a row
  unit_t* lds = reinterpret_cast<unit_t*>(smem);

  // Workgroup -> tile.  Hardware deals consecutive workgroup ids round-robin over the 8
  // XCDs; remap so that each XCD walks a contiguous range of tiles (tiles that share a
  // weight panel then share one L2).
  const int w = blockIdx.x;
  const int slot = (w % 8) * p.chunks + w / 8;
  if (slot >= p.total) return;
  // Which of a tile's split ranges this workgroup takes.  Dense layers: the splits of one tile
  // are neighbours.  Convolution weight gradients (CONV == 2): the tiles of one split range are
  // neighbours instead, because they all read the same rows of the output gradient and
  // overlapping pixels of the image -- as neighbours they find them in their XCD's L2 (with
  // the other order a 64 -> 64 channel layer at 4 x 128 x 32 x 32 pixels fetched 1.0 GB per
  // launch from HBM, four times what it reads).
  const int tiles_all = p.total / p.splits;
  const int split = CONV == 2 ? slot / tiles_all : slot % p.splits;
  const int logical = CONV == 2 ? slot % tiles_all : slot / p.splits;
  // Inside a replica, tiles go in bands of GROUP_M tile rows, m fastest inside a band: the
  // workgroups running together then cover a compact block of the output, and the operand
  // panels they share stay within one XCD's L2.
  constexpr int GROUP_M = 8;
  const int per_rep = p.tilesM * p.tilesN;
  const int bat = logical / per_rep;
  const int t = logical - bat * per_rep;
  const int band = t / (GROUP_M * p.tilesN);
  const int first_m = band * GROUP_M;
  const int gsize = p.tilesM - first_m < GROUP_M ? p.tilesM - first_m : GROUP_M;
  const int tin = t - band * GROUP_M * p.tilesN;
  const int tm_idx = first_m + tin % gsize;
  const int tn_idx = tin / gsize;
  const int m0 = tm_idx * BM, n0 = tn_idx * BN;

  const T* A = reinterpret_cast<const T*>(p.A) + (long long)bat * p.strideA;
  const T* B = reinterpret_cast<const T*>(p.B) + (long long)bat * p.strideB;
  const unsigned bytesA = CONV == 1 ? (unsigned)(p.M * p.cm.C) * sizeof(T)
                                    : (unsigned)((A_KMAJOR ? p.M : p.Kd) * p.ldA) * sizeof(T);
  const unsigned bytesB = CONV == 2 ? (unsigned)(p.Kd * p.cm.C) * sizeof(T)
                                    : (unsigned)((B_KMAJOR ? p.N : p.Kd) * p.ldB) * sizeof(T);
  const __amdgpu_buffer_rsrc_t rsrcA = make_rsrc(A, bytesA);
  const __amdgpu_buffer_rsrc_t rsrcB = make_rsrc(B, bytesB);

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

  TileLoader<T, BM, A_KMAJOR, BKU, CONV == 1 ? 1 : 0> la;
  TileLoader<T, BN, B_KMAJOR, BKU, CONV == 2 ? 2 : 0> lb;
  if constexpr (CONV == 1) la.prepare(p.cm, m0, p.M, tid);
  if constexpr (CONV == 2) lb.prepare(p.cm, n0, p.N, tid);
  auto load_a = [&](int k0u) {
    if constexpr (CONV == 1) la.load_unfolded(rsrcA, p.cm, k0u, p.Kd, tid);
    else la.load(rsrcA, p.ldA, m0, p.M, k0u, p.Kd, tid);
  };
  auto load_b = [&](int k0u) {
    if constexpr (CONV == 2) lb.load_unfolded(rsrcB, p.cm, k0u, p.Kd, tid);
    else lb.load(rsrcB, p.ldB, n0, p.N, k0u, p.Kd, tid);
  };
  constexpr int NKC = BKU / 2;                        // k-chunks (one MFMA depth each) per k-step
  constexpr int ND = TM + TN;                         // LDS fragment reads per k-chunk
  constexpr int NM = TM * TN * (UE == 4 ? 4 : 1);     // MFMAs per k-chunk
  constexpr int NW = TileLoader<T, BM, A_KMAJOR, BKU>::NSTORE +
                     TileLoader<T, BN, B_KMAJOR, BKU>::NSTORE;   // LDS writes per k-step
  constexpr int NV = TileLoader<T, BM, A_KMAJOR, BKU>::NREG +
                     TileLoader<T, BN, B_KMAJOR, BKU>::NREG;     // global loads per k-step
  const int ksteps_all = (p.Kd + BKU * UE - 1) / (BKU * UE);
  const int kbeg = split * p.steps_per_split;                  // first k-step of this split
  const int ksteps = ksteps_all - kbeg < p.steps_per_split ? ksteps_all - kbeg : p.steps_per_split;
  const int kb = kbeg * BKU;

  // LDS read positions of this lane (k-unit `h` of each k-chunk is added per chunk)
  int posA[TM], posB[TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
    posA[i] = h * (BM + PAD) + (BF16MATH ? swz_half(wm0 + i * 32 + l32) : swz<UE>(wm0 + i * 32 + l32));
#pragma unroll
  for (int j = 0; j < TN; ++j)
    posB[j] = A_UNITS + h * (BN + PAD) + (BF16MATH ? swz_half(wn0 + j * 32 + l32) : swz<UE>(wn0 + j * 32 + l32));

  unit_t fa[2][TM], fb[2][TN];
  auto read_frags = [&](const unit_t* stage, int kc, int buf) {
#pragma unroll
    for (int i = 0; i < TM; ++i) fa[buf][i] = stage[posA[i] + kc * 2 * (BM + PAD)];
#pragma unroll
    for (int j = 0; j < TN; ++j) fb[buf][j] = stage[posB[j] + kc * 2 * (BN + PAD)];
  };
  u32x2 ha[TM], hb[TN];     // BF16MATH: the even chunk's operands, rounded, waiting for the odd one
  auto mfma_chunk = [&](int buf) {
    if constexpr (BF16MATH) {
      // chunk parity equals the fragment buffer index (an even number of chunks per k-step)
      if (buf == 0) {
#pragma unroll
        for (int i = 0; i < TM; ++i) ha[i] = fa[0][i];
#pragma unroll
        for (int j = 0; j < TN; ++j) hb[j] = fb[0][j];
      } else {
        u32x4 qa[TM], qb[TN];
#pragma unroll
        for (int i = 0; i < TM; ++i) qa[i] = u32x4{ha[i][0], ha[i][1], fa[1][i][0], fa[1][i][1]};
#pragma unroll
        for (int j = 0; j < TN; ++j) qb[j] = u32x4{hb[j][0], hb[j][1], fb[1][j][0], fb[1][j][1]};
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
          for (int j = 0; j < TN; ++j)
            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, qb[j]),
                                                                __builtin_bit_cast(bf16x8, qa[i]),
                                                                acc[i][j], 0, 0, 0);
      }
    } else {
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) {
          if constexpr (UE == 4) {
            const f32x4 a = __builtin_bit_cast(f32x4, fa[buf][i]);
            const f32x4 b = __builtin_bit_cast(f32x4, fb[buf][j]);
#pragma unroll
            for (int e = 0; e < 4; ++e)
              acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(b[e], a[e], acc[i][j], 0, 0, 0);
          } else {
            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
                __builtin_bit_cast(bf16x8, fb[buf][j]), __builtin_bit_cast(bf16x8, fa[buf][i]),
                acc[i][j], 0, 0, 0);
          }
        }
    }
  };

  // Software pipeline.  At the top of k-step ks: LDS buffer ks&1 holds tile ks, the registers
  // of the loaders hold tile ks+1 (in flight), fragment buffer 0 holds k-chunk 0 of tile ks.
  //   chunks 0..NKC-2: read the next chunk's fragments while the MFMAs of this one run; in
  //                    the last of them also write tile ks+1 to the other LDS buffer;
  //   barrier;
  //   chunk NKC-1:     its MFMAs cover the barrier, the fragment reads of tile ks+1 and the
  //                    issue of the global loads of tile ks+2.
  // The scheduling hints fix that interleaving; left alone, the compiler sinks every LDS read
  // next to its first use and the single wavefront per SIMD stalls on each one.
  load_a(kb);
  load_b(kb);
  la.store(lds, tid);
  lb.store(lds + A_UNITS, tid);
  load_a(kb + BKU);      // past the end: reads as zeros
  load_b(kb + BKU);
  __syncthreads();
  read_frags(lds, 0, 0);

  for (int ks = 0; ks + 1 < ksteps; ++ks) {
    const unit_t* cur = lds + (ks & 1) * STAGE_UNITS;
    unit_t* nxt = lds + ((ks + 1) & 1) * STAGE_UNITS;
#pragma unroll
    for (int kc = 0; kc + 1 < NKC; ++kc) {
      read_frags(cur, kc + 1, (kc + 1) & 1);
      mfma_chunk(kc & 1);
      if (kc + 2 == NKC) {
        la.store(nxt, tid);
        lb.store(nxt + A_UNITS, tid);
        if constexpr (!BF16MATH) Pipeline<ND, NW, 0x200, NM>::run();
      } else {
        if constexpr (!BF16MATH) Pipeline<ND, 0, 0, NM>::run();
      }
    }
    __syncthreads();
    read_frags(nxt, 0, 0);
    mfma_chunk((NKC - 1) & 1);
    load_a(kb + (ks + 2) * BKU);
    load_b(kb + (ks + 2) * BKU);
    if constexpr (!BF16MATH) Pipeline<ND, NV, 0x020, NM>::run();
  }
  {
    const unit_t* cur = lds + ((ksteps - 1) & 1) * STAGE_UNITS;
#pragma unroll
    for (int kc = 0; kc < NKC; ++kc) {
      if (kc + 1 < NKC) read_frags(cur, kc + 1, (kc + 1) & 1);
      mfma_chunk(kc & 1);
      if constexpr (!BF16MATH) if (kc + 1 < NKC) Pipeline<ND, 0, 0, NM>::run();
    }
  }
  __syncthreads();

  // Epilogue.  With the swapped MFMA roles, accumulator element e of a 32x32 tile belongs to
  // row m = l32 and column n = (e/4)*8 + h*4 + e%4.  Stores straight from that layout would
  // scatter 16-byte pieces over 32 rows per instruction; instead the tile is passed through
  // LDS (now free) 64 rows at a time and written out as whole rows, consecutive lanes on
  // consecutive 16 bytes, which is also how bias and the ReLU mask are read.
  const bool split_mode = p.splits > 1;     // raw partial sums; bias/ReLU/mask wait for the reduce
  TC* C = split_mode ? reinterpret_cast<TC*>(p.partial + (long long)split * p.strideSplit +
                                             (long long)bat * p.M * p.ldP)
                     : reinterpret_cast<TC*>(p.C) + (long long)bat * p.strideC;
  const int ldC = split_mode ? p.ldP : p.ldC;
  const float* bias = p.bias ? p.bias + (long long)bat * p.strideBias : nullptr;
  const float* bias_dir = p.bias_dir ? p.bias_dir + (long long)bat * p.strideBias : nullptr;
  const float bias_sc = p.bias_dir ? p.bias_scale[bat] : 0.f;
  const T* mask = p.mask ? reinterpret_cast<const T*>(p.mask) + (long long)bat * p.strideMask
                         : nullptr;
  const bool has_bias = !split_mode && (p.epilogue == EPI_BIAS || p.epilogue == EPI_BIAS_RELU);
  const bool relu = !split_mode && p.epilogue == EPI_BIAS_RELU;
  const bool masked = !split_mode && p.epilogue == EPI_MASK;
  typedef typename Pack<TC>::vec cvec;
  typedef typename Pack<T>::vec mvec;
  constexpr int PITCH = BN + 4;                 // floats; +4 keeps the 16-byte writes off one bank
  constexpr int LANES_PER_ROW = BN / 4;         // lanes that cover one row of the tile
  constexpr int ROWS_PER_PASS = kThreads / LANES_PER_ROW;
  float* stage = reinterpret_cast<float*>(smem);
  const int c4 = (tid % LANES_PER_ROW) * 4;     // first of this lane's 4 columns (read-out phase)
  const int rsub = tid / LANES_PER_ROW;
  const int n = n0 + c4;
  float ssq = 0.f;                              // squares of what this thread stores
  f32x4 bv = {0.f, 0.f, 0.f, 0.f};
  if (has_bias) {
#pragma unroll
    for (int r = 0; r < 4; ++r)
      if (n + r < p.N) {
        bv[r] = bias[n + r];
        if (bias_dir) bv[r] = bv[r] + bias_sc * bias_dir[n + r];   // bias of the perturbed point
      }
  }
#pragma unroll
  for (int i = 0; i < TM; ++i) {
    // rows of this pass: for each of the two wave rows, its i-th 32-row strip
    const int lrow = (wave >> 1) * 32 + l32;
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        f32x4 v;
#pragma unroll
        for (int r = 0; r < 4; ++r) v[r] = acc[i][j][q * 4 + r];
        *reinterpret_cast<f32x4*>(stage + lrow * PITCH + wn0 + j * 32 + q * 8 + h * 4) = v;
      }
    __syncthreads();
#pragma unroll
    for (int pass = 0; pass < 64 / ROWS_PER_PASS; ++pass) {
      const int rr = pass * ROWS_PER_PASS + rsub;
      const int m = m0 + (rr >> 5) * (BM / 2) + i * 32 + (rr & 31);
      if (m < p.M && n < p.N) {
        f32x4 v = *reinterpret_cast<const f32x4*>(stage + rr * PITCH + c4);
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          v[r] += bv[r];
          if (relu) v[r] = v[r] > 0.f ? v[r] : 0.f;
        }
        if (n + 3 < p.N) {
          if (masked) {
            const mvec mk = *reinterpret_cast<const mvec*>(mask + (long long)m * p.ldMask + n);
            const T* me = reinterpret_cast<const T*>(&mk);
#pragma unroll
            for (int r = 0; r < 4; ++r)
              if (!(widen(me[r]) > 0.f)) v[r] = 0.f;
          }
          *reinterpret_cast<cvec*>(C + (long long)m * ldC + n) = Pack<TC>::from(v);
          ssq += (v[0] * v[0] + v[1] * v[1]) + (v[2] * v[2] + v[3] * v[3]);
        } else {
#pragma unroll
          for (int r = 0; r < 4; ++r)
            if (n + r < p.N) {
              float o = v[r];
              if (masked && !(widen(mask[(long long)m * p.ldMask + n + r]) > 0.f)) o = 0.f;
              C[(long long)m * ldC + n + r] = Pack<TC>::one(o);
              ssq += o * o;
            }
        }
      }
    }
    if (i + 1 < TM) __syncthreads();
  }
  if (p.sumsq != nullptr && !split_mode) {
    const double tot = workgroup_sum((double)ssq);
    if (tid == 0) p.sumsq[(long long)bat * p.strideSumsq + t] = tot;
  }
}

// Sums the split-K partials in a fixed order and applies the epilogue the GEMM skipped.
// Grid: x over groups of 256 of the M * ldP/4 vector words of one replica, y = replica.  A
// workgroup is LANES x 256 threads; with LANES = 4, thread (lane group q, word) adds the partials q, q+4, q+8, ...
// of its word (four chains of loads in flight instead of one: with up to 128 partials the
// single chain was the whole run time), the four sums are combined through LDS as
// ((q0 + q1) + (q2 + q3)), and lane group 0 finishes the word.
// (With fewer than 8 partials one chain is short enough: LANES = 1, a workgroup of 256.)
template <int LANES>
__global__ __launch_bounds__(kThreads * LANES) void splitk_reduce_kernel(GemmParams p) {
  constexpr int kReduceLanes = LANES;
  __shared__ f32x4 part[LANES > 1 ? LANES - 1 : 1][kThreads];
  __shared__ double wsum[kThreads / 64];
  const int n4 = p.ldP / 4;
  const long long per_rep = (long long)p.M * n4;
  const int word = threadIdx.x % kThreads, q = threadIdx.x / kThreads;
  const long long idx = (long long)blockIdx.x * kThreads + word;
  const int bat = blockIdx.y;
  const bool live = idx < per_rep;
  const int c = live ? (int)(idx % n4) * 4 : 0;
  const int m = live ? (int)(idx / n4) : 0;
  const long long row = (long long)bat * p.M + m;
  f32x4 v = {0.f, 0.f, 0.f, 0.f};
  if (live && c < p.N)
    for (int s = q; s < p.splits; s += kReduceLanes)
      v += *reinterpret_cast<const f32x4*>(p.partial + (long long)s * p.strideSplit + row * p.ldP + c);
  if constexpr (LANES > 1) {
    if (q > 0) part[q - 1][word] = v;
    __syncthreads();
  }
  float ssq = 0.f;
  if (q == 0 && live && c < p.N) {
    if constexpr (LANES == 4) v = (v + part[0][word]) + (part[1][word] + part[2][word]);
    const bool has_bias = p.epilogue == EPI_BIAS || p.epilogue == EPI_BIAS_RELU;
    float* C = reinterpret_cast<float*>(p.C) + (long long)bat * p.strideC + (long long)m * p.ldC;
    const float* mask = p.mask ? reinterpret_cast<const float*>(p.mask) +
                                     (long long)bat * p.strideMask + (long long)m * p.ldMask
                               : nullptr;
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      const int n = c + r;
      if (n >= p.N) break;
      float o = v[r];
      if (has_bias) {
        float bv = p.bias[(long long)bat * p.strideBias + n];
        if (p.bias_dir) bv = bv + p.bias_scale[bat] * p.bias_dir[(long long)bat * p.strideBias + n];
        o += bv;
      }
      if (p.epilogue == EPI_BIAS_RELU) o = o > 0.f ? o : 0.f;
      if (p.epilogue == EPI_MASK && !(mask[n] > 0.f)) o = 0.f;
      C[n] = o;
      ssq += o * o;
    }
  }
  if (p.sumsq != nullptr) {
    // lane group 0 is the first four wavefronts: lanes by xor-shuffle, then the four in turn
    if (q == 0) {
      double t = (double)ssq;
#pragma unroll
      for (int off = 32; off > 0; off >>= 1) t += __shfl_xor(t, off, 64);
      if ((word & 63) == 0) wsum[word >> 6] = t;
    }
    __syncthreads();
    if (threadIdx.x == 0)
      p.sumsq[(long long)bat * p.strideSumsq + blockIdx.x] = (wsum[0] + wsum[1]) + (wsum[2] + wsum[3]);
  }
}

// Tile shape and split of the contraction for one GEMM, chosen from measurements on MI355X at
// the workload shapes: the forward GEMM (both operands k-major, few staging registers) runs
// best as 256x128 tiles with two workgroups per compute unit; the GEMMs with transposing loads
// as 256x256 with one; smaller tiles only where the larger ones would leave compute units
// idle.  When even 64x64 or 128x128 tiles give fewer than two workgroups per compute unit and
// the contraction is long (fp32 configurations with small batches), the contraction is split
// so that every SIMD has work; the partial sums are reduced in a fixed order.
struct Plan {
  int bm, bn, bku;
  int splits, steps_per_split, ldP;
  size_t ws_bytes;
};

// 64x64 tiles replace 128x128 ones when they compute less than this fraction of the work
constexpr double kSmallTileGain = 0.88;

Plan make_plan(const GemmDesc& d, int tile_override) {
  auto tiles = [&](int bm, int bn) {
    return (long long)((d.M + bm - 1) / bm) * ((d.N + bn - 1) / bn) * d.batch;
  };
  Plan pl{64, 64, 8, 1, 0, 0, 0};
  const bool kk = d.a_kmajor && d.b_kmajor;
  if (tile_override == 1) { pl.bm = 256; pl.bn = 256; }
  else if (tile_override == 2) { pl.bm = 256; pl.bn = 128; pl.bku = 4; }
  else if (tile_override == 4) { pl.bm = 128; pl.bn = 128; }
  else if (tile_override == 5) { pl.bm = 64; pl.bn = 64; }
  else if (d.unfold || d.bf16_math) {   // instantiated for the two smaller tiles only
    // (for the weight gradients, few output tiles and a split contraction, the smaller tile
    // measured faster: 71 us against 84 us at M = 128, N = 576, 8192 pixels, 4 replicas;
    // k-steps twice as deep, and 128x64 / 64x128 tiles, changed nothing)
    if (d.M >= 128 && d.N >= 128 && tiles(128, 128) >= (d.bf16_math ? 192 : 512)) { pl.bm = 128; pl.bn = 128; }
    else if (d.bf16_math && d.unfold == 2 && d.M >= 128 && d.N >= 128 && d.Kd >= 2048) { pl.bm = 128; pl.bn = 128; }
    // extents such as 160 or 320 channels fill only part of their last 128-wide tile; when the
    // 64-wide tiling computes enough less, it wins although its tiles run a little slower
    // (WRN-16x10, fp32: forward 50.7 -> 45.1 ms, dX 52.5 -> 46.6 ms per step; with bf16 products
    // the small tile is too much slower: 51.9 -> 63 ms per step, so not there)
    if (pl.bm == 128 && !d.bf16_math &&
        (double)tiles(64, 64) * 64 * 64 < kSmallTileGain * (double)tiles(128, 128) * 128 * 128) {
      pl.bm = 64; pl.bn = 64;
    }
  }
  else if (kk && d.M >= 256 && d.N >= 128 && tiles(256, 128) >= 512) { pl.bm = 256; pl.bn = 128; pl.bku = 4; }
  else if (d.M >= 256 && d.N >= 256 && tiles(256, 256) >= 512) { pl.bm = 256; pl.bn = 256; }
  else if (d.M >= 128 && d.N >= 128 && tiles(128, 128) >= 256) { pl.bm = 128; pl.bn = 128; }
  const int ue = d.in_bf16 ? 8 : 4;
  const int ksteps = (d.Kd + pl.bku * ue - 1) / (pl.bku * ue);
  pl.steps_per_split = ksteps;
  const long long nt = tiles(pl.bm, pl.bn);
  // 512 workgroups measured best for the dense layers' shapes; the convolutions' weight
  // gradients (tiny outputs, contractions of 10^4..10^5) want more of the small tiles in
  // flight: a wavefront of a 64x64 tile has little work per k-step to cover the latency of
  // its next loads with
  const int target = (pl.bm == 64 && d.Kd >= 8192) ? 2048 : 512;
  if (!d.out_bf16 && !d.in_bf16 && nt < target && ksteps >= 8) {
    int want = (int)((target + nt - 1) / nt);
    int cap = ksteps / 4;
    int sp = want < cap ? want : cap;
    // up to 16 splits; more only for the very long contractions of convolution weight
    // gradients (batch x image rows), whose outputs are a handful of tiles
    const int most = d.Kd >= 131072 ? 128 : (d.Kd >= 32768 ? 64 : (d.Kd >= 8192 ? 32 : 16));
    if (sp > most) sp = most;
    if (sp > 1) {
      pl.steps_per_split = (ksteps + sp - 1) / sp;
      pl.splits = (ksteps + pl.steps_per_split - 1) / pl.steps_per_split;
      pl.ldP = (d.N + 3) / 4 * 4;
      pl.ws_bytes = (size_t)pl.splits * d.batch * d.M * pl.ldP * 4;
    }
  }
  return pl;
}

template <typename T, typename TC, int BM, int BN, int BKU, bool AK, bool BK_, int CONV = 0,
          bool BF16MATH = false>
int launch_one(const GemmParams& p0, hipStream_t s, int* sumsq_slots) {
  constexpr int OCC = (BM * BN >= 256 * 256) ? 1 : 2;
  GemmParams p = p0;
  p.tilesM = (p.M + BM - 1) / BM;
  p.tilesN = (p.N + BN - 1) / BN;
  p.total = p.tilesM * p.tilesN * p.batch * p.splits;
  p.chunks = (p.total + 7) / 8;
  const size_t loop_smem = BF16MATH ? (size_t)2 * BKU * ((BM + 2) + (BN + 2)) * 8
                                    : (size_t)2 * BKU * ((BM + 1) + (BN + 1)) * 16;
  const size_t epi_smem = (size_t)64 * (BN + 4) * 4;
  const size_t smem = loop_smem > epi_smem ? loop_smem : epi_smem;
  auto kern = gemm_kernel<T, TC, BM, BN, BKU, AK, BK_, OCC, CONV, BF16MATH>;
  static std::atomic<bool> attr_set{false};   // per instantiation; setting it twice is harmless
  if (!attr_set.load(std::memory_order_relaxed)) {
    if (hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                            hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem) != hipSuccess)
      return -1;
    attr_set.store(true, std::memory_order_relaxed);
  }
  kern<<<p.chunks * 8, kThreads, smem, s>>>(p);
  int slots = p.tilesM * p.tilesN;
  if (p.splits > 1) {
    const long long per_rep = (long long)p.M * (p.ldP / 4);
    slots = (int)((per_rep + kThreads - 1) / kThreads);
    if (p.splits >= 8)
      splitk_reduce_kernel<4><<<dim3((unsigned)slots, (unsigned)p.batch), kThreads * 4, 0, s>>>(p);
    else
      splitk_reduce_kernel<1><<<dim3((unsigned)slots, (unsigned)p.batch), kThreads, 0, s>>>(p);
  }
  if (sumsq_slots) *sumsq_slots = slots;
  return 0;
}

template <typename T, typename TC, bool AK, bool BK_>
int launch_tiled(const GemmParams& p, const Plan& pl, hipStream_t s, int* slots) {
  if (pl.bm == 256 && pl.bn == 128) return launch_one<T, TC, 256, 128, 4, AK, BK_>(p, s, slots);
  if (pl.bm == 256) return launch_one<T, TC, 256, 256, 8, AK, BK_>(p, s, slots);
  if (pl.bm == 128) return launch_one<T, TC, 128, 128, 8, AK, BK_>(p, s, slots);
  return launch_one<T, TC, 64, 64, 8, AK, BK_>(p, s, slots);
}

template <typename T, typename TC>
int launch_layout(const GemmDesc& d, const GemmParams& p, const Plan& pl, hipStream_t s, int* slots) {
  if (d.bf16_math) {
    const bool big = pl.bm == 128;
    if (d.unfold == 1) {
      if (!(d.a_kmajor && d.b_kmajor)) return -1;
      return big ? launch_one<T, TC, 128, 128, 8, true, true, 1, true>(p, s, slots)
                 : launch_one<T, TC, 64, 64, 8, true, true, 1, true>(p, s, slots);
    }
    if (d.unfold == 2) {
      if (d.a_kmajor || d.b_kmajor) return -1;
      return big ? launch_one<T, TC, 128, 128, 8, false, false, 2, true>(p, s, slots)
                 : launch_one<T, TC, 64, 64, 8, false, false, 2, true>(p, s, slots);
    }
    if (d.a_kmajor && d.b_kmajor)
      return big ? launch_one<T, TC, 128, 128, 8, true, true, 0, true>(p, s, slots)
                 : launch_one<T, TC, 64, 64, 8, true, true, 0, true>(p, s, slots);
    if (d.a_kmajor && !d.b_kmajor)
      return big ? launch_one<T, TC, 128, 128, 8, true, false, 0, true>(p, s, slots)
                 : launch_one<T, TC, 64, 64, 8, true, false, 0, true>(p, s, slots);
    if (!d.a_kmajor && !d.b_kmajor)
      return big ? launch_one<T, TC, 128, 128, 8, false, false, 0, true>(p, s, slots)
                 : launch_one<T, TC, 64, 64, 8, false, false, 0, true>(p, s, slots);
    return -1;
  }
  if (d.unfold == 1) {
    if (!(d.a_kmajor && d.b_kmajor)) return -1;
    if (pl.bm == 128) return launch_one<T, TC, 128, 128, 8, true, true, 1>(p, s, slots);
    return launch_one<T, TC, 64, 64, 8, true, true, 1>(p, s, slots);
  }
  if (d.unfold == 2) {
    if (d.a_kmajor || d.b_kmajor) return -1;
    if (pl.bm == 128) return launch_one<T, TC, 128, 128, 8, false, false, 2>(p, s, slots);
    return launch_one<T, TC, 64, 64, 8, false, false, 2>(p, s, slots);
  }
  if (d.a_kmajor && d.b_kmajor) return launch_tiled<T, TC, true, true>(p, pl, s, slots);
  if (d.a_kmajor && !d.b_kmajor) return launch_tiled<T, TC, true, false>(p, pl, s, slots);
  if (!d.a_kmajor && !d.b_kmajor) return launch_tiled<T, TC, false, false>(p, pl, s, slots);
  return -1;
}

}  // namespace

size_t gemm_splitk_bytes(const GemmDesc& d) { return make_plan(d, 0).ws_bytes; }

// Smallest tiles are 64x64; a split-K reduce uses one workgroup per 256 vector words of
// [M][N rounded up to 4].
int gemm_sumsq_capacity(int M, int N) {
  const long long tiles = (long long)((M + 63) / 64) * ((N + 63) / 64);
  const long long words = ((long long)M * ((N + 3) / 4) + kThreads - 1) / kThreads;
  return (int)(tiles > words ? tiles : words);
}

int launch_gemm(const GemmDesc& d, hipStream_t s, int* sumsq_slots) {
  // bf16 operands live in the blocked layout and have their own kernel; this file's kernel
  // serves the fp32 configurations
  if (d.in_bf16) return (d.unfold || d.bf16_math) ? -1 : launch_gemm_bf16(d, 0, s, sumsq_slots);
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
  p.partial = nullptr; p.strideSplit = 0; p.ldP = 0; p.splits = 1; p.steps_per_split = 1 << 30;
  p.sumsq = d.sumsq; p.strideSumsq = d.sumsq_stride;
  if (d.M <= 0 || d.N <= 0 || d.Kd <= 0 || d.batch <= 0) return -1;
  p.cm = ConvMap{0, 1, 1, 1.f, 1.f, 0};
  if (d.unfold) {
    // a k-step (32 floats) must lie inside one tap; pixel indices must be exact in fp32; the
    // contraction (mode 1) or the column extent (mode 2) is the unfolded width 9 C
    const long long pixels = d.unfold == 1 ? d.M : d.Kd;
    if (d.unfold_C % 32 || d.unfold_H < 1 || d.unfold_W < 1 ||
        pixels % ((long long)d.unfold_H * d.unfold_W) || pixels >= (1 << 24) ||
        pixels * d.unfold_C * 4 >= 0x7FFFFFF0LL || (d.unfold == 1 ? d.Kd : d.N) != 9 * d.unfold_C)
      return -1;
    p.cm = ConvMap{d.unfold_C, d.unfold_H, d.unfold_W, 1.f / (float)d.unfold_W, 1.f / (float)d.unfold_H,
                   (d.unfold_W % 4 == 0 && 32 % d.unfold_W == 0) ? 32 / d.unfold_W : 0};
  }
  // 16-byte units: pitches must be multiples of 8 elements and bases 16-byte aligned.
  if ((d.ldA % 8) || (d.ldB % 8) || (d.ldC % 8) || ((uintptr_t)d.A & 15) ||
      ((uintptr_t)d.B & 15) || ((uintptr_t)d.C & 15))
    return -1;
  if (d.epilogue == EPI_MASK && ((d.ldMask % 8) || ((uintptr_t)d.mask & 15))) return -1;
  // buffer-load offsets are 32-bit byte offsets inside one replica's operand
  const long long es = d.in_bf16 ? 2 : 4;
  const long long rowsA = d.a_kmajor ? d.M : d.Kd, rowsB = d.b_kmajor ? d.N : d.Kd;
  if (rowsA * d.ldA * es >= 0x7FFFFFF0LL || rowsB * d.ldB * es >= 0x7FFFFFF0LL) return -1;
  if ((d.strideA % 4) || (d.strideB % 4) || (d.strideC % 4)) return -1;
  if (d.out_bf16) return -1;
  Plan pl = make_plan(d, 0);
  if (pl.splits > 1 && d.splitk_ws != nullptr && d.splitk_bytes >= pl.ws_bytes &&
      ((uintptr_t)d.splitk_ws & 15) == 0) {
    p.partial = d.splitk_ws;
    p.splits = pl.splits;
    p.steps_per_split = pl.steps_per_split;
    p.ldP = pl.ldP;
    p.strideSplit = (long long)d.batch * d.M * pl.ldP;
  }
  return launch_layout<float, float>(d, p, pl, s, sumsq_slots);
}

}  // namespace lsam
