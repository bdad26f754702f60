// bf16 replica GEMMs with an LDS ring fed by direct global->LDS loads.
//
// Same contract as the generic kernel (C[m,n] = sum_k A(m,k) B(n,k), operands k-major or
// m-major, batched over replicas) for bf16 operands stored in the blocked layout of b32s.h.
// No operand passes through registers on its way to LDS:
//   * every thread issues `buffer_load_dwordx4 ... lds` instructions; a wavefront instruction
//     copies 1 KiB of global memory to 1 KiB of LDS in lane order.  Because a tile is a run
//     of whole 2 KiB blocks in that layout, the LDS image of a tile is a plain copy of it.
//   * k-major fragments are one 128-bit LDS read; m-major fragments are two transposing LDS
//     reads (ds_read_b64_tr_b16: within 16 lanes, lanes 4j..4j+3 address row j of a 4x16
//     block and lane i receives column i), which delivers exactly the MFMA operand layout, so
//     neither weights nor activations need a transposed copy or a register shuffle.
//   * a k-step is 32 deep (two MFMA depths); NSTAGE-1 k-steps are in flight behind the one
//     being multiplied (~96 KiB per compute unit), which is what hides HBM latency with a
//     single wavefront per SIMD.  Each stage is its own LDS array so that the compiler's
//     wait-count tracking can tell them apart; the wait that orders a stage's arrival before
//     the workgroup barrier is explicit.
#include "engine.h"
#include "b32s.h"

namespace lsam {
namespace {

constexpr int kThreads = 256;
constexpr int BK = 32;        // bf16 elements of k per stage

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __attribute__((address_space(3))) unsigned char lds_byte;

struct Bf16GemmParams {
  const char* A; long long strideA; int ldA;
  const char* B; long long strideB; int ldB;
  char* C; long long strideC; int ldC;
  int M, N, Kd, batch;
  int tilesM, tilesN, total, chunks;
  int epilogue;
  const float* bias; long long strideBias;
  const float* bias_dir; const float* bias_scale;
  const char* mask; long long strideMask; int ldMask;
  int cbA, cbB, cbC, cbMask;          // column blocks of the stored A, B, C (bf16 out) and mask
  unsigned bytesA, bytesB;            // size of one replica's stored A and B
  double* sumsq; long long strideSumsq;   // optional: sum of squares of each tile's results
  // EPI_STEP kernels: the sampler step taken on the result instead of storing it
  float* fx; float* fv; float* fS; const float* fy;
  unsigned short* fshadow; long long strideShadow; int cbShadow;
  float lr, mu; int nesterov;
  ReplicaScalars lam;
  const int* frestart;                    // per-replica marks: 1 = the sum S starts afresh (may be null)
  // EPI_ASCEND kernels: x (same addressing as the result), the per-replica scale rho/(||g||+gamma),
  // and the operand copy that receives bf16(x + scale g) (fshadow, strideShadow, cbShadow above)
  const float* ax; const float* ascale;
  int mode;                               // EPI_* the launch asks for
  // EPI_STORE with a plain fp32 result only: the contraction is cut into ksplit pieces, each
  // taken by a workgroup of its own; piece j of replica k writes its partial result at
  // C + k * strideC + j * strideSplit (elements)
  int ksplit; long long strideSplit;
};

// s_waitcnt immediate: vmcnt = vm (0..63), lgkmcnt = lgkm (0..15), expcnt untouched.
constexpr int waitcnt(int vm, int lgkm) {
  return (vm & 0xF) | ((vm >> 4) << 14) | (0x7 << 4) | ((lgkm & 0xF) << 8);
}

__device__ __forceinline__ __amdgpu_buffer_rsrc_t make_rsrc(const void* base, unsigned bytes) {
  const unsigned long long a = reinterpret_cast<unsigned long long>(base);
  const unsigned lo = __builtin_amdgcn_readfirstlane((unsigned)a);
  const unsigned hi = __builtin_amdgcn_readfirstlane((unsigned)(a >> 32));
  void* ptr = reinterpret_cast<void*>(((unsigned long long)hi << 32) | lo);
  return __builtin_amdgcn_make_buffer_rsrc(ptr, 0, __builtin_amdgcn_readfirstlane(bytes),
                                           0x00020000);
}

// One operand tile of R rows (of the output) by BK of k, as it lives in one LDS stage.
template <int R, bool KMAJOR, int NFRAG>
struct Operand {
  static constexpr int BYTES = R * BK * 2;
  static constexpr int NLOAD = BYTES / (kThreads * 16);       // load instructions per thread
  static constexpr int NREAD = KMAJOR ? NFRAG : 2 * NFRAG;    // LDS reads per MFMA depth
  unsigned goff[NLOAD];       // global byte offset of this lane's 16 bytes at k-step 0
  unsigned kstep;             // bytes from one k-step to the next
  unsigned lds_slot0;         // LDS byte offset (in the tile) of the wavefront's first 1 KiB chunk
  // LDS byte offsets of the reads of fragment 0, [depth][half]; fragment t lies t*2048 bytes
  // further (one 32-row or 32-column block) for both kinds of operand.
  unsigned rd[1][2][KMAJOR ? 1 : 2];

  // cblocks: column blocks of the stored matrix; row0: first output row (or column) of the
  // tile, a multiple of 32; wrow0: first row of this wavefront's part inside the tile.
  __device__ __forceinline__ void init(int cblocks, int row0, int wrow0, int tid) {
    const int lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int l32 = lane & 31, h = lane >> 5;
    lds_slot0 = (unsigned)(wave * NLOAD) * 1024u;
#pragma unroll
    for (int j = 0; j < NLOAD; ++j) {
      const unsigned tb = (unsigned)(wave * NLOAD + j) * 1024u + (unsigned)lane * 16u;  // byte in the tile
      if constexpr (KMAJOR) {
        // R/32 blocks, one per 32 rows, `cblocks` blocks apart in memory
        goff[j] = ((unsigned)(row0 >> 5) + (tb >> 11)) * (unsigned)cblocks * 2048u + (tb & 2047u);
      } else {
        // R/32 consecutive blocks of one block row
        goff[j] = (unsigned)(row0 >> 5) * 2048u + tb;
      }
    }
    kstep = KMAJOR ? 2048u : (unsigned)cblocks * 2048u;
#pragma unroll
    for (int kc = 0; kc < 2; ++kc) {
      if constexpr (KMAJOR) {
        const int r = wrow0 + l32;
        const int ku = kc * 2 + h;
        rd[0][kc][0] = (unsigned)(r * 64 + ((ku ^ ((r >> 2) & 3)) * 16));
      } else {
        const int il = lane & 15, gq = lane >> 4;
#pragma unroll
        for (int kk = 0; kk < 2; ++kk) {
          const int kr = kc * 16 + (gq >> 1) * 8 + kk * 4 + (il >> 2);
          const int col = wrow0 + (gq & 1) * 16 + 4 * (il & 3);
          rd[0][kc][kk] = (unsigned)((col >> 5) * 2048 + kr * 64 +
                                     ((((col & 31) >> 3) ^ ((kr >> 2) & 3)) << 4) + (col & 7) * 2);
        }
      }
    }
  }

  // Moves the tile's first k-step `first` steps into the contraction.
  __device__ __forceinline__ void skip(int first) {
#pragma unroll
    for (int j = 0; j < NLOAD; ++j) goff[j] += (unsigned)first * kstep;
  }

  // Requests k-step `ks` of the tile into `tile`.  A step at or past `ksteps` is sent out of
  // range on purpose: the stage then fills with zeros, which add nothing when multiplied.
  __device__ __forceinline__ void issue(__amdgpu_buffer_rsrc_t rsrc, lds_byte* tile, int ks,
                                        int ksteps) const {
    const unsigned adv = ks < ksteps ? (unsigned)ks * kstep : 0x7FFFFFF0u;
#pragma unroll
    for (int j = 0; j < NLOAD; ++j)
      __builtin_amdgcn_raw_ptr_buffer_load_lds(
          rsrc, (__attribute__((address_space(3))) void*)(tile + lds_slot0 + j * 1024), 16,
          ks < ksteps ? goff[j] + adv : 0x7FFFFFF0u, 0, 0, 0);
  }

  __device__ __forceinline__ void read(const lds_byte* tile, int kc, u32x4 (&f)[NFRAG]) const {
#pragma unroll
    for (int t = 0; t < NFRAG; ++t) {
      if constexpr (KMAJOR) {
        f[t] = *reinterpret_cast<const __attribute__((address_space(3))) u32x4*>(
            tile + rd[0][kc][0] + t * 2048);
      } else {
#if defined(__HIP_DEVICE_COMPILE__)
        const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
            (__attribute__((address_space(3))) s16x4*)(tile + rd[0][kc][0] + t * 2048));
        const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
            (__attribute__((address_space(3))) s16x4*)(tile + rd[0][kc][1] + t * 2048));
        const u32x2 l2 = __builtin_bit_cast(u32x2, lo), h2 = __builtin_bit_cast(u32x2, hi);
        f[t][0] = l2[0]; f[t][1] = l2[1]; f[t][2] = h2[0]; f[t][3] = h2[1];
#endif
      }
    }
  }
};

template <int MASK, int N, int M, int I>
struct Interleave {
  static __device__ __forceinline__ void run() {
    constexpr int ops = N * (I + 1) / M - N * I / M;
    if constexpr (ops > 0) __builtin_amdgcn_sched_group_barrier(MASK, ops, 0);
    __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
    if constexpr (I + 1 < M) Interleave<MASK, N, M, I + 1>::run();
  }
};

template <typename TC> struct Out;
template <> struct Out<float> {
  typedef f32x4 vec;
  static __device__ __forceinline__ vec from(const f32x4& v) { return v; }
  static __device__ __forceinline__ float one(float v) { return v; }
};
template <> struct Out<__bf16> {
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

// What the epilogue does with the result tile.
//   EPI_STORE   store it (with bias / ReLU / mask as the launch says, optionally the sum of squares)
//   EPI_STEP    weight gradient at the perturbed point: take the sampler step on it
//   EPI_SUMSQ   weight gradient of the first pass: only its sum of squares is wanted
//   EPI_ASCEND  weight gradient of the first pass, recomputed once the norm is known: write
//               the operand copy of the perturbed weights, bf16(x + scale * g)
enum { EPI_STORE = 0, EPI_STEP = 1, EPI_SUMSQ = 2, EPI_ASCEND = 3 };
constexpr int kStepGroup = 4;      // EPI_STEP: side of the tile groups an XCD takes through all replicas
constexpr int kAscendBand = 2;    // EPI_ASCEND: tile rows of the band all XCDs share

template <typename TC, int BM, int BN, int NSTAGE, bool A_KMAJOR, bool B_KMAJOR, int OCC, int MODE = EPI_STORE>
__global__ __launch_bounds__(kThreads, OCC) void gemm_bf16_kernel(Bf16GemmParams p) {
  static_assert(MODE == EPI_STORE || sizeof(TC) == 4, "the fused epilogues work on fp32 results");
  static_assert(NSTAGE == 3 || NSTAGE == 4, "ring of 3 or 4 stages");
  constexpr int TM = BM / 64, TN = BN / 64;
  constexpr int A_BYTES = BM * BK * 2, B_BYTES = BN * BK * 2;
  constexpr int EPI_PITCH = BN / 2 + 4;                       // epilogue staging pitch (floats)
  constexpr int EPI_BYTES = 2 * 32 * EPI_PITCH * 4;           // two wavefronts stage in one array
  constexpr int STAGE_BYTES = A_BYTES + B_BYTES > EPI_BYTES ? A_BYTES + B_BYTES : EPI_BYTES;
  __shared__ __attribute__((aligned(1024))) unsigned char st0[STAGE_BYTES];
  __shared__ __attribute__((aligned(1024))) unsigned char st1[STAGE_BYTES];
  __shared__ __attribute__((aligned(1024))) unsigned char st2[STAGE_BYTES];
  __shared__ __attribute__((aligned(1024))) unsigned char st3[NSTAGE == 4 ? STAGE_BYTES : 1024];

  const int w = blockIdx.x;
  int bat, m0, n0, t_in = 0, piece = 0;
  if constexpr (MODE == EPI_STEP) {
    // The step reads the centre y, which all replicas share: an XCD takes whole groups of
    // kStepGroup x kStepGroup tiles and works through the replicas of one group before it
    // moves to the next, so that the group's piece of y comes from memory once per XCD and
    // from that XCD's L2 for the other replicas (replica-major order fetched it once per
    // replica).  chunks = workgroups per XCD = groups per XCD * batch * tiles per group; tiles
    // of a ragged group that fall outside the matrix leave at once.
    constexpr int G = kStepGroup;
    const int idx = w / 8;
    const int t = idx % (G * G);
    const int rest = idx / (G * G);
    bat = rest % p.batch;
    const int group = (rest / p.batch) * 8 + (w % 8);
    const int groupsN = (p.tilesN + G - 1) / G;
    const int tm = (group / groupsN) * G + t % G, tn = (group % groupsN) * G + t / G;
    if (tm >= p.tilesM || tn >= p.tilesN) return;
    m0 = tm * BM; n0 = tn * BN;
  } else if constexpr (MODE == EPI_ASCEND) {
    // All XCDs work in the same replica and band of kAscendBand tile rows, XCD x on the column
    // tiles n = 8 n' + x: the row panels of the first operand are then wanted by all eight at
    // about the same time instead of by one XCD per replica (8.9-9.0 against 9.2-9.3 ms per
    // step of the largest configuration; bands of 1 to 4 tile rows alike, 8 and 16 slower).
    // chunks = workgroups per XCD = batch * tilesM * ceil(tilesN / 8).
    constexpr int GROUP_M = kAscendBand;
    const int x = w % 8, idx = w / 8;
    const int tn8 = (p.tilesN + 7) / 8;
    const int per_rep = p.tilesM * tn8;
    bat = idx / per_rep;
    if (bat >= p.batch) return;
    t_in = idx - bat * per_rep;
    const int band = t_in / (GROUP_M * tn8);
    const int first_m = band * GROUP_M;
    const int gsize = p.tilesM - first_m < GROUP_M ? p.tilesM - first_m : GROUP_M;
    const int tin = t_in - band * GROUP_M * tn8;
    const int tn = (tin / gsize) * 8 + x;
    if (tn >= p.tilesN) return;
    m0 = (first_m + tin % gsize) * BM; n0 = tn * BN;
  } else {
    const int logical = (w % 8) * p.chunks + w / 8;    // contiguous tile range per XCD
    if (logical >= p.total) return;
    constexpr int GROUP_M = 8;
    const int per_rep = p.tilesM * p.tilesN;
    bat = logical / per_rep;
    t_in = logical - bat * per_rep;
    if (p.ksplit > 1) {                                // (replica, piece of the contraction)
      piece = bat % p.ksplit;
      bat /= p.ksplit;
    }
    const int band = t_in / (GROUP_M * p.tilesN);
    const int first_m = band * GROUP_M;
    const int gsize = p.tilesM - first_m < GROUP_M ? p.tilesM - first_m : GROUP_M;
    const int tin = t_in - band * GROUP_M * p.tilesN;
    m0 = (first_m + tin % gsize) * BM; n0 = (tin / gsize) * BN;
  }

  const __bf16* A = reinterpret_cast<const __bf16*>(p.A) + (long long)bat * p.strideA;
  const __bf16* B = reinterpret_cast<const __bf16*>(p.B) + (long long)bat * p.strideB;
  const __amdgpu_buffer_rsrc_t rsrcA = make_rsrc(A, p.bytesA);
  const __amdgpu_buffer_rsrc_t rsrcB = make_rsrc(B, p.bytesB);

  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  const int wm0 = (wave >> 1) * (BM / 2), wn0 = (wave & 1) * (BN / 2);
  const int l32 = lane & 31, h = lane >> 5;

  Operand<BM, A_KMAJOR, TM> oa;
  Operand<BN, B_KMAJOR, TN> ob;
  oa.init(p.cbA, m0, wm0, tid);
  ob.init(p.cbB, n0, wn0, tid);
  constexpr int NL = Operand<BM, A_KMAJOR, TM>::NLOAD + Operand<BN, B_KMAJOR, TN>::NLOAD;
  constexpr int ND = Operand<BM, A_KMAJOR, TM>::NREAD + Operand<BN, B_KMAJOR, TN>::NREAD;
  constexpr int NM = TM * TN;

  f32x16 acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

  u32x4 fa[2][TM], fb[2][TN];
  auto mfma_chunk = [&](int buf) {
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int j = 0; j < TN; ++j)
        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
            __builtin_bit_cast(bf16x8, fb[buf][j]), __builtin_bit_cast(bf16x8, fa[buf][i]),
            acc[i][j], 0, 0, 0);
  };

  int ksteps = (p.Kd + BK - 1) / BK;           // the stored operands are zero-padded to 32
  if (p.ksplit > 1) {
    // this workgroup's piece of the contraction: k-steps [first, first + ksteps), possibly none
    const int per = (ksteps + p.ksplit - 1) / p.ksplit;
    const int first = piece * per;
    ksteps = ksteps - first < per ? ksteps - first : per;
    if (ksteps < 0) ksteps = 0;
    oa.skip(first);
    ob.skip(first);
  }
  lds_byte* s0 = (lds_byte*)st0;
  lds_byte* s1 = (lds_byte*)st1;
  lds_byte* s2 = (lds_byte*)st2;
  lds_byte* s3 = (lds_byte*)st3;

  // Tiles past the last k-step are still requested (as zeros), which keeps the number of
  // loads in flight, and so the wait counts, the same in every step, and lets the loop run
  // in whole rounds of the four stages.
  oa.issue(rsrcA, s0, 0, ksteps); ob.issue(rsrcB, s0 + A_BYTES, 0, ksteps);
  oa.issue(rsrcA, s1, 1, ksteps); ob.issue(rsrcB, s1 + A_BYTES, 1, ksteps);
  oa.issue(rsrcA, s2, 2, ksteps); ob.issue(rsrcB, s2 + A_BYTES, 2, ksteps);
  if constexpr (NSTAGE == 4) {
    oa.issue(rsrcA, s3, 3, ksteps); ob.issue(rsrcB, s3 + A_BYTES, 3, ksteps);
  }
  __builtin_amdgcn_s_waitcnt(waitcnt((NSTAGE - 1) * NL, 15));   // tile 0 has landed (this wavefront's part)
  asm volatile("" ::: "memory");
  __builtin_amdgcn_s_barrier();
  asm volatile("" ::: "memory");
  oa.read(s0, 0, fa[0]);
  ob.read(s0 + A_BYTES, 0, fb[0]);

  // One k-step on stage CUR; NEXT holds the following tile; the tile NSTAGE steps ahead is
  // requested into CUR as soon as every wavefront has taken its last fragment out of it.
#define LSAM_GEMM_STEP(CUR, NEXT)                                                         \
  {                                                                                       \
    oa.read(CUR, 1, fa[1]);                                                               \
    ob.read(CUR + A_BYTES, 1, fb[1]);                                                     \
    mfma_chunk(0);                                                                        \
    Interleave<0x100, ND, NM, 0>::run();                                                  \
    __builtin_amdgcn_s_waitcnt(waitcnt((NSTAGE - 2) * NL, 0));                            \
    asm volatile("" ::: "memory");                                                        \
    __builtin_amdgcn_s_barrier();                                                         \
    asm volatile("" ::: "memory");                                                        \
    oa.issue(rsrcA, CUR, ks + NSTAGE, ksteps);                                            \
    ob.issue(rsrcB, CUR + A_BYTES, ks + NSTAGE, ksteps);                                  \
    oa.read(NEXT, 0, fa[0]);                                                              \
    ob.read(NEXT + A_BYTES, 0, fb[0]);                                                    \
    mfma_chunk(1);                                                                        \
    Interleave<0x120, ND + NL, NM, 0>::run();                                             \
    ++ks;                                                                                 \
  }

  for (int ks = 0; ks < ksteps;) {
    LSAM_GEMM_STEP(s0, s1)
    LSAM_GEMM_STEP(s1, s2)
    if constexpr (NSTAGE == 3) {
      LSAM_GEMM_STEP(s2, s0)
    } else {
      LSAM_GEMM_STEP(s2, s3)
      LSAM_GEMM_STEP(s3, s0)
    }
  }
#undef LSAM_GEMM_STEP
  __builtin_amdgcn_s_waitcnt(waitcnt(0, 0));           // nothing may still be writing LDS
  asm volatile("" ::: "memory");
  __builtin_amdgcn_s_barrier();
  asm volatile("" ::: "memory");

  // Epilogue.  Element e of a 32x32 accumulator tile is row m = l32, column
  // n = (e/4)*8 + h*4 + e%4 (the MFMA was issued with rows <- B, columns <- A); storing from
  // that layout would scatter 16-byte pieces over 32 rows per instruction.  Each wavefront
  // instead passes its own 32-row strips through a private piece of LDS (no workgroup
  // barrier: LDS operations of one wavefront complete in order) and writes them out as row
  // segments, consecutive lanes on consecutive 16 bytes; bias and the ReLU mask are read the
  // same way.
  TC* C = reinterpret_cast<TC*>(p.C) + (long long)bat * p.strideC + (long long)piece * p.strideSplit;
  const float* bias = p.bias ? p.bias + (long long)bat * p.strideBias : nullptr;
  const float* bias_dir = p.bias_dir ? p.bias_dir + (long long)bat * p.strideBias : nullptr;
  const float bias_sc = p.bias_dir ? p.bias_scale[bat] : 0.f;
  const __bf16* mask = p.mask ? reinterpret_cast<const __bf16*>(p.mask) + (long long)bat * p.strideMask
                              : nullptr;
  const bool has_bias = p.epilogue == EPI_BIAS || p.epilogue == EPI_BIAS_RELU;
  const bool relu = p.epilogue == EPI_BIAS_RELU;
  const bool masked = p.epilogue == EPI_MASK;
  typedef typename Out<TC>::vec cvec;
  constexpr int WN = BN / 2;                       // columns of a wavefront's part
  constexpr int LANES_PER_ROW = WN / 4;
  constexpr int ROWS_PER_PASS = 64 / LANES_PER_ROW;
  float* stage = reinterpret_cast<float*>((wave >> 1) ? st1 : st0) + (wave & 1) * (32 * EPI_PITCH);
  const int c4 = (lane % LANES_PER_ROW) * 4;
  const int rsub = lane / LANES_PER_ROW;
  const int n = n0 + wn0 + c4;
  float ssq = 0.f;                                 // squares of what this thread stores
  if constexpr (MODE == EPI_STEP) {
    // The sampler step on the tile instead of storing it.  x, v, S, y and the operand copy are
    // addressed as buffers (one descriptor each, a 32-bit byte offset per lane), so that rows
    // past M and columns past N fall out of range -- their loads return zero and their stores
    // are dropped -- and no lane needs 64-bit addresses.  The state of NB passes is requested
    // in one go before the first result is touched: a wavefront then has 4 NB 16-byte loads
    // per lane in flight instead of 4, which lets these streams run at memory speed rather
    // than at one round trip per pass.  Columns N..ldC-1 are row padding holding zeros in x, v,
    // S and y; the gradient there is zero (the operands are zero-padded), so they stay zero.
    float lam = 0.f;
    // picked with constant indices: a variable index would move the whole argument block to
    // private memory
#pragma unroll
    for (int k = 0; k < kMaxK; ++k)
      if (k == bat) lam = p.lam.v[k];
    constexpr int PASSES = 32 / ROWS_PER_PASS;
    // (the 128x128 tile, 64 accumulator registers per lane, has room for all eight passes of a
    // strip at once: 27.3 / 26.9 against 27.8 / 27.0 ms per step with four)
    constexpr int DEPTH = BM * BN <= 128 * 128 ? 8 : 4;
    constexpr int NB = PASSES < DEPTH ? PASSES : DEPTH;
    constexpr unsigned kOut = 0x7FFFFFF0u;          // beyond every buffer: ignored by the hardware
    // Cache policies (bit 0 sc0, bit 1 nt, bit 4 sc1).  The state is read once and written
    // once per step: loads are non-temporal, stores non-temporal and written through at system
    // scope, the 8-byte stores of the operand copy as well.  Measured on 16 x [8192 x 8192]
    // layers: no hints 31.6 ms per step of the largest configuration, nt on loads and state
    // stores 30.2, nt + write-through on every store 28.7 (sc0 alone 31.6, sc1 alone 28.8).
    constexpr int NT = 2;
    constexpr int WT = 2 | 1 | 16;
    const unsigned wbytes = (unsigned)p.M * (unsigned)p.ldC * 4u;
    const __amdgpu_buffer_rsrc_t rx = make_rsrc(p.fx + (long long)bat * p.strideC, wbytes);
    const __amdgpu_buffer_rsrc_t rv = make_rsrc(p.fv + (long long)bat * p.strideC, wbytes);
    const __amdgpu_buffer_rsrc_t rs = make_rsrc(p.fS + (long long)bat * p.strideC, wbytes);
    const __amdgpu_buffer_rsrc_t ry = make_rsrc(p.fy, wbytes);
    const __amdgpu_buffer_rsrc_t rw = make_rsrc(p.fshadow + (long long)bat * p.strideShadow,
                                                (unsigned)(b32s_blocks(p.M) * p.cbShadow) * 2048u);
    const bool col_ok = n < p.N;
    const unsigned rowbytes = (unsigned)p.ldC * 4u;
    const unsigned off0 = (unsigned)(m0 + wm0 + rsub) * rowbytes + (unsigned)n * 4u;
    // a replica served by the last center update starts its sum afresh: S is not read (its
    // loads go out of range and return zeros)
    const bool fresh = p.frestart != nullptr && p.frestart[bat] == 1;
#pragma unroll
    for (int i = 0; i < TM; ++i) {
#pragma unroll
      for (int j = 0; j < TN; ++j)
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          f32x4 v;
#pragma unroll
          for (int r = 0; r < 4; ++r) v[r] = acc[i][j][q * 4 + r];
          *reinterpret_cast<f32x4*>(stage + l32 * EPI_PITCH + j * 32 + q * 8 + h * 4) = v;
        }
#pragma unroll
      for (int pb = 0; pb < PASSES; pb += NB) {
        u32x4 xv[NB], vv[NB], sv[NB], yv[NB];
#pragma unroll
        for (int u = 0; u < NB; ++u) {
          const unsigned off = col_ok ? off0 + (unsigned)(i * 32 + (pb + u) * ROWS_PER_PASS) * rowbytes : kOut;
          xv[u] = __builtin_amdgcn_raw_buffer_load_b128(rx, off, 0, NT);
          vv[u] = __builtin_amdgcn_raw_buffer_load_b128(rv, off, 0, NT);
          sv[u] = __builtin_amdgcn_raw_buffer_load_b128(rs, fresh ? kOut : off, 0, NT);
          yv[u] = __builtin_amdgcn_raw_buffer_load_b128(ry, off, 0, 0);
        }
#pragma unroll
        for (int u = 0; u < NB; ++u) {
          const int rr = (pb + u) * ROWS_PER_PASS + rsub;
          const int m = m0 + wm0 + i * 32 + rr;
          const unsigned off = col_ok ? off0 + (unsigned)(i * 32 + (pb + u) * ROWS_PER_PASS) * rowbytes : kOut;
          const f32x4 gv = *reinterpret_cast<const f32x4*>(stage + rr * EPI_PITCH + c4);
          f32x4 xe = __builtin_bit_cast(f32x4, xv[u]), ve = __builtin_bit_cast(f32x4, vv[u]);
          f32x4 se = __builtin_bit_cast(f32x4, sv[u]);
          const f32x4 ye = __builtin_bit_cast(f32x4, yv[u]);
#pragma unroll
          for (int r = 0; r < 4; ++r) {
            float a = xe[r], b = ve[r], c = se[r];
            sampler_step(gv[r], ye[r], lam, p.lr, p.mu, p.nesterov, 0.f, a, b, c);
            xe[r] = a; ve[r] = b; se[r] = c;
          }
          __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(u32x4, xe), rx, off, 0, WT);
          __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(u32x4, ve), rv, off, 0, WT);
          __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(u32x4, se), rs, off, 0, WT);
          const unsigned woff = (col_ok && m < p.M) ? (unsigned)b32s_offset(m, n, p.cbShadow) * 2u : kOut;
          __builtin_amdgcn_raw_buffer_store_b64(Out<__bf16>::from(xe), rw, woff, 0, WT);
        }
      }
    }
    return;
  }
  if constexpr (MODE == EPI_ASCEND) {
    // The ascent perturbation on the tile: x~ = x + scale g, rounded to bf16 into the operand
    // copy.  Same buffer addressing; x is streamed in once, four passes at a time.
    constexpr int PASSES = 32 / ROWS_PER_PASS;
    constexpr int NB = PASSES < 4 ? PASSES : 4;
    constexpr unsigned kOut = 0x7FFFFFF0u;
    const __amdgpu_buffer_rsrc_t rx = make_rsrc(p.ax + (long long)bat * p.strideC,
                                                (unsigned)p.M * (unsigned)p.ldC * 4u);
    const __amdgpu_buffer_rsrc_t rw = make_rsrc(p.fshadow + (long long)bat * p.strideShadow,
                                                (unsigned)(b32s_blocks(p.M) * p.cbShadow) * 2048u);
    const float sc = p.ascale[bat];
    const bool col_ok = n < p.N;
    const unsigned rowbytes = (unsigned)p.ldC * 4u;
    const unsigned off0 = (unsigned)(m0 + wm0 + rsub) * rowbytes + (unsigned)n * 4u;
#pragma unroll
    for (int i = 0; i < TM; ++i) {
#pragma unroll
      for (int j = 0; j < TN; ++j)
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          f32x4 v;
#pragma unroll
          for (int r = 0; r < 4; ++r) v[r] = acc[i][j][q * 4 + r];
          *reinterpret_cast<f32x4*>(stage + l32 * EPI_PITCH + j * 32 + q * 8 + h * 4) = v;
        }
#pragma unroll
      for (int pb = 0; pb < PASSES; pb += NB) {
        u32x4 xv[NB];
#pragma unroll
        for (int u = 0; u < NB; ++u) {
          const unsigned off = col_ok ? off0 + (unsigned)(i * 32 + (pb + u) * ROWS_PER_PASS) * rowbytes : kOut;
          xv[u] = __builtin_amdgcn_raw_buffer_load_b128(rx, off, 0, 2);
        }
#pragma unroll
        for (int u = 0; u < NB; ++u) {
          const int rr = (pb + u) * ROWS_PER_PASS + rsub;
          const int m = m0 + wm0 + i * 32 + rr;
          const f32x4 gv = *reinterpret_cast<const f32x4*>(stage + rr * EPI_PITCH + c4);
          f32x4 xe = __builtin_bit_cast(f32x4, xv[u]);
#pragma unroll
          for (int r = 0; r < 4; ++r) xe[r] = ascent_point(xe[r], sc, gv[r]);
          const unsigned woff = (col_ok && m < p.M) ? (unsigned)b32s_offset(m, n, p.cbShadow) * 2u : kOut;
          // non-temporal and written through, like the step's stores of the same copy (with a
          // plain store here the step kernel that later overwrites the copy ran 4 % slower)
          __builtin_amdgcn_raw_buffer_store_b64(Out<__bf16>::from(xe), rw, woff, 0, 2 | 1 | 16);
        }
      }
    }
    return;
  }
  f32x4 bv = {0.f, 0.f, 0.f, 0.f};
  if (has_bias) {
#pragma unroll
    for (int r = 0; r < 4; ++r)
      if (n + r < p.N) {
        bv[r] = bias[n + r];
        if (bias_dir) bv[r] = bv[r] + bias_sc * bias_dir[n + r];
      }
  }
#pragma unroll
  for (int i = 0; i < TM; ++i) {
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        f32x4 v;
#pragma unroll
        for (int r = 0; r < 4; ++r) v[r] = acc[i][j][q * 4 + r];
        *reinterpret_cast<f32x4*>(stage + l32 * EPI_PITCH + j * 32 + q * 8 + h * 4) = v;
      }
#pragma unroll
    for (int pass = 0; pass < 32 / ROWS_PER_PASS; ++pass) {
      const int rr = pass * ROWS_PER_PASS + rsub;
      const int m = m0 + wm0 + i * 32 + rr;
      f32x4 v = *reinterpret_cast<const f32x4*>(stage + rr * EPI_PITCH + c4);
      if (m < p.M && n < p.N) {
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          v[r] += bv[r];
          if (relu) v[r] = v[r] > 0.f ? v[r] : 0.f;
        }
        // bf16 results and the mask are in the blocked layout (4 consecutive n share a unit);
        // fp32 results are row-major
        long long coff;
        if constexpr (sizeof(TC) == 2) coff = b32s_offset(m, n, p.cbC);
        else coff = (long long)m * p.ldC + n;
        const long long moff = masked ? b32s_offset(m, n, p.cbMask) : 0;
        if (n + 3 < p.N) {
          if (masked) {
            const u32x2 mk = *reinterpret_cast<const u32x2*>(mask + moff);
            const __bf16* me = reinterpret_cast<const __bf16*>(&mk);
#pragma unroll
            for (int r = 0; r < 4; ++r)
              if (!(static_cast<float>(me[r]) > 0.f)) v[r] = 0.f;
          }
          if constexpr (MODE != EPI_SUMSQ)
            __builtin_nontemporal_store(Out<TC>::from(v), reinterpret_cast<cvec*>(C + coff));
          ssq += (v[0] * v[0] + v[1] * v[1]) + (v[2] * v[2] + v[3] * v[3]);
        } else {
#pragma unroll
          for (int r = 0; r < 4; ++r)
            if (n + r < p.N) {
              float o = v[r];
              if (masked && !(static_cast<float>(mask[moff + r]) > 0.f)) o = 0.f;
              if constexpr (MODE != EPI_SUMSQ) C[coff + r] = Out<TC>::one(o);
              ssq += o * o;
            }
        }
      }
    }
  }
  if (p.sumsq != nullptr) {
    // fixed order: lanes by xor-shuffle, then the four wavefronts in turn
    __shared__ double part[4];
    double tot = (double)ssq;
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) tot += __shfl_xor(tot, off, 64);
    if (lane == 0) part[wave] = tot;
    __syncthreads();
    if (tid == 0) p.sumsq[(long long)bat * p.strideSumsq + t_in] = (part[0] + part[1]) + (part[2] + part[3]);
  }
}

// Every specialisation that can be launched is instantiated explicitly (the host-side launch
// stubs of implicit instantiations of this kernel were not all emitted by the compiler).
#define LSAM_INSTANTIATE(TC, AK, BK_)                                                         \
  template __global__ void gemm_bf16_kernel<TC, 256, 256, 4, AK, BK_, 1>(Bf16GemmParams);      \
  template __global__ void gemm_bf16_kernel<TC, 256, 128, 3, AK, BK_, 2>(Bf16GemmParams);      \
  template __global__ void gemm_bf16_kernel<TC, 128, 128, 4, AK, BK_, 2>(Bf16GemmParams);
LSAM_INSTANTIATE(float, true, true)
LSAM_INSTANTIATE(float, true, false)
LSAM_INSTANTIATE(float, false, false)
LSAM_INSTANTIATE(__bf16, true, true)
LSAM_INSTANTIATE(__bf16, true, false)
LSAM_INSTANTIATE(__bf16, false, false)
#undef LSAM_INSTANTIATE
#define LSAM_INSTANTIATE_MODE(M)                                                                         \
  template __global__ void gemm_bf16_kernel<float, 256, 256, 4, false, false, 1, M>(Bf16GemmParams);  \
  template __global__ void gemm_bf16_kernel<float, 256, 128, 3, false, false, 2, M>(Bf16GemmParams);  \
  template __global__ void gemm_bf16_kernel<float, 128, 128, 4, false, false, 2, M>(Bf16GemmParams);
LSAM_INSTANTIATE_MODE(EPI_STEP)
LSAM_INSTANTIATE_MODE(EPI_SUMSQ)
LSAM_INSTANTIATE_MODE(EPI_ASCEND)
#undef LSAM_INSTANTIATE_MODE

template <typename TC, int BM, int BN, int NSTAGE, bool AK, bool BK_>
int launch_one(const Bf16GemmParams& p0, hipStream_t s, int* slots) {
  constexpr int OCC = (BM * BN >= 256 * 256) ? 1 : 2;
  Bf16GemmParams p = p0;
  p.tilesM = (p.M + BM - 1) / BM;
  p.tilesN = (p.N + BN - 1) / BN;
  p.total = p.tilesM * p.tilesN * p.batch * p.ksplit;
  p.chunks = (p.total + 7) / 8;
  if constexpr (sizeof(TC) == 4 && !AK && !BK_) {
    // the fused epilogues exist for weight-gradient launches (both operands m-major) only
    if (p.mode == EPI_STEP) {
      const long long groups = (long long)((p.tilesM + kStepGroup - 1) / kStepGroup) *
                               ((p.tilesN + kStepGroup - 1) / kStepGroup);
      const long long per_xcd = (groups + 7) / 8 * p.batch * kStepGroup * kStepGroup;
      if (per_xcd * 8 >= (1ll << 31)) return -1;
      p.chunks = (int)per_xcd;
      gemm_bf16_kernel<TC, BM, BN, NSTAGE, AK, BK_, OCC, EPI_STEP><<<p.chunks * 8, kThreads, 0, s>>>(p);
      if (slots) *slots = 0;
      return 0;
    }
    if (p.mode == EPI_ASCEND) {
      const long long per_xcd = (long long)p.batch * p.tilesM * ((p.tilesN + 7) / 8);
      if (per_xcd * 8 >= (1ll << 31)) return -1;
      p.chunks = (int)per_xcd;
      gemm_bf16_kernel<TC, BM, BN, NSTAGE, AK, BK_, OCC, EPI_ASCEND><<<p.chunks * 8, kThreads, 0, s>>>(p);
      if (slots) *slots = 0;
      return 0;
    }
    if (p.mode == EPI_SUMSQ) {
      gemm_bf16_kernel<TC, BM, BN, NSTAGE, AK, BK_, OCC, EPI_SUMSQ><<<p.chunks * 8, kThreads, 0, s>>>(p);
      if (slots) *slots = p.tilesM * p.tilesN;
      return 0;
    }
  }
  if (p.mode != EPI_STORE) return -1;
  gemm_bf16_kernel<TC, BM, BN, NSTAGE, AK, BK_, OCC><<<p.chunks * 8, kThreads, 0, s>>>(p);
  if (slots) *slots = p.tilesM * p.tilesN;
  return 0;
}

template <typename TC, bool AK, bool BK_>
int launch_tiled(const Bf16GemmParams& p, int tile, hipStream_t s, int* slots) {
  if (tile == 256) return launch_one<TC, 256, 256, 4, AK, BK_>(p, s, slots);
  if (tile == 2) return launch_one<TC, 256, 128, 3, AK, BK_>(p, s, slots);
  return launch_one<TC, 128, 128, 4, AK, BK_>(p, s, slots);
}

template <typename TC>
int launch_layout(const GemmDesc& d, const Bf16GemmParams& p, int tile, hipStream_t s, int* slots) {
  if (d.a_kmajor && d.b_kmajor) return launch_tiled<TC, true, true>(p, tile, s, slots);
  if (d.a_kmajor && !d.b_kmajor) return launch_tiled<TC, true, false>(p, tile, s, slots);
  if (!d.a_kmajor && !d.b_kmajor) return launch_tiled<TC, false, false>(p, tile, s, slots);
  return -1;
}

}  // namespace

// All bf16 GEMMs of the MLP path come here; operands, bf16 results and the mask are in the
// blocked layout.  Returns 0 after a launch, -1 if the description is not usable.
int launch_gemm_bf16(const GemmDesc& d, int tile_override, hipStream_t s, int* sumsq_slots) {
  if (!d.in_bf16 || !d.b32s) return -1;
  if (d.M <= 0 || d.N <= 0 || d.Kd <= 0 || d.batch <= 0) return -1;
  auto tiles = [&](int bm, int bn) {
    return (long long)((d.M + bm - 1) / bm) * ((d.N + bn - 1) / bn) * d.batch;
  };
  // By measurement on MI355X: 256x256 tiles (one workgroup per compute unit) once there are
  // enough of them to fill the chip twice -- except for the weight gradient with a short
  // contraction (batch < 1024), where a second workgroup per unit hides the per-tile start-up
  // and write-out (1.28 against 1.49 ms for 16 x [8192 x 8192] at batch 512); 256x128 tiles
  // with a three-stage ring (two workgroups per unit) when the batch still gives 256 rows;
  // 128x128 otherwise.  A fifth ring stage (all 160 KiB of LDS) measured no faster than four.
  int tile = 128;
  if (tile_override == 1) tile = 256;
  else if (tile_override == 2) tile = 2;
  else if (tile_override == 4) tile = 128;
  // (the input gradient, whose weights are read through transposing LDS reads, also prefers
  // 256x128: 9.3 against 9.8 ms per step of the largest configuration; the forward pass
  // 256x256: 9.5 against 9.9)
  else if (d.M >= 256 && d.N >= 256 && tiles(256, 256) >= 512 &&
           (d.Kd >= 1024 ? (d.b_kmajor || !d.a_kmajor) : d.a_kmajor && d.b_kmajor)) tile = 256;
  else if (d.M >= 256 && d.N >= 128 && tiles(256, 128) >= 256) tile = 2;
  // The step epilogue streams seven arrays per tile; there the 128x128 tile (two workgroups per
  // compute unit, four-stage ring) measured best: 27.0-27.8 ms per step of the largest
  // configuration against 28.7-29.9 for 256x128 tiles, two workgroups per unit (and 30.3 for
  // 256x256); the ascent epilogue, one array in and one out, keeps the choice above (9.1 against
  // 9.6 ms with 128x128).
  if (d.fuse != nullptr && tile_override == 0) tile = 128;
  const int kpad = (d.Kd + 31) / 32 * 32;
  // stored shapes: k-major [rows][k], m-major [k][rows]
  const long long blocksA = d.a_kmajor ? (long long)b32s_blocks(d.M) * d.cbA : (long long)b32s_blocks(kpad) * d.cbA;
  const long long blocksB = d.b_kmajor ? (long long)b32s_blocks(d.N) * d.cbB : (long long)b32s_blocks(kpad) * d.cbB;
  // 32-bit byte offsets: the farthest block a lane can name (8 tiles of rows, 4 k-steps past
  // the end) must stay below 2^31
  if ((blocksA + (long long)(16 + 8) * d.cbA + 64) * 2048 >= 0x7FFFFFF0LL ||
      (blocksB + (long long)(16 + 8) * d.cbB + 64) * 2048 >= 0x7FFFFFF0LL)
    return -1;
  if (d.a_kmajor ? d.cbA < b32s_blocks(d.Kd) : d.cbA < b32s_blocks(d.M)) return -1;
  if (d.b_kmajor ? d.cbB < b32s_blocks(d.Kd) : d.cbB < b32s_blocks(d.N)) return -1;
  if (((uintptr_t)d.A & 15) || ((uintptr_t)d.B & 15) || (d.strideA % 1024) || (d.strideB % 1024))
    return -1;
  Bf16GemmParams p;
  p.A = (const char*)d.A; p.strideA = d.strideA; p.ldA = d.ldA;
  p.B = (const char*)d.B; p.strideB = d.strideB; p.ldB = d.ldB;
  p.C = (char*)d.C; p.strideC = d.strideC; p.ldC = d.ldC;
  p.M = d.M; p.N = d.N; p.Kd = d.Kd; p.batch = d.batch;
  p.tilesM = p.tilesN = p.total = p.chunks = 0;
  p.epilogue = d.epilogue;
  p.bias = d.bias; p.strideBias = d.strideBias;
  p.bias_dir = d.bias_dir; p.bias_scale = d.bias_scale;
  p.mask = (const char*)d.mask; p.strideMask = d.strideMask; p.ldMask = d.ldMask;
  p.cbA = d.cbA; p.cbB = d.cbB; p.cbC = d.cbC; p.cbMask = d.cbMask;
  p.bytesA = (unsigned)(blocksA * 2048);
  p.bytesB = (unsigned)(blocksB * 2048);
  p.sumsq = d.out_bf16 ? nullptr : d.sumsq;
  p.strideSumsq = d.sumsq_stride;
  p.fx = nullptr; p.frestart = nullptr;
  p.mode = EPI_STORE;
  const bool plain_f32 = !d.out_bf16 && d.epilogue == EPI_PLAIN && (d.ldC % 4) == 0 && (d.strideC % 4) == 0;
  p.ksplit = 1; p.strideSplit = 0;
  if (d.ksplit > 1) {
    // partial results of a split contraction: plain fp32 stores and nothing else
    if (!plain_f32 || d.sumsq != nullptr || d.fuse != nullptr || d.ascend != nullptr || d.sumsq_only ||
        d.ksplit > 64 || (d.split_stride % 4) != 0 || tiles(128, 128) * d.ksplit >= (1ll << 28))
      return -1;
    p.ksplit = d.ksplit; p.strideSplit = d.split_stride;
  }
  // 32-bit byte offsets inside one replica's W_l, rows of a ragged last tile included
  const bool offsets_fit = ((long long)d.M + 256) * d.ldC * 4 < 0x7FFFFFF0LL;
  if (d.fuse != nullptr) {
    const SamplerFusion& f = *d.fuse;
    // 16-byte accesses at k * strideC + m * ldC + n with n a multiple of 4
    if (!plain_f32 || !offsets_fit || ((uintptr_t)f.x & 15) || ((uintptr_t)f.v & 15) ||
        ((uintptr_t)f.S & 15) || ((uintptr_t)f.y & 15) || ((uintptr_t)f.shadow & 7) ||
        f.cbShadow < b32s_blocks(d.N) || (long long)b32s_blocks(d.M) * f.cbShadow * 2048 >= 0x7FFFFFF0LL)
      return -1;
    p.fx = f.x; p.fv = f.v; p.fS = f.S; p.fy = f.y;
    p.fshadow = f.shadow; p.strideShadow = f.shadow_stride; p.cbShadow = f.cbShadow;
    p.lr = f.lr; p.mu = f.mu; p.nesterov = f.nesterov;
    p.lam = f.lam;
    p.frestart = f.restart;
    p.sumsq = nullptr;
    p.mode = EPI_STEP;
  } else if (d.ascend != nullptr) {
    const AscentFusion& f = *d.ascend;
    if (!plain_f32 || !offsets_fit || ((uintptr_t)f.x & 15) || ((uintptr_t)f.shadow & 7) || !f.scale ||
        f.cbShadow < b32s_blocks(d.N) || (long long)b32s_blocks(d.M) * f.cbShadow * 2048 >= 0x7FFFFFF0LL)
      return -1;
    p.ax = f.x; p.ascale = f.scale;
    p.fshadow = f.shadow; p.strideShadow = f.shadow_stride; p.cbShadow = f.cbShadow;
    p.sumsq = nullptr;
    p.mode = EPI_ASCEND;
  } else if (d.sumsq_only) {
    if (!plain_f32 || d.sumsq == nullptr) return -1;
    p.mode = EPI_SUMSQ;
  }
  return d.out_bf16 ? launch_layout<__bf16>(d, p, tile, s, sumsq_slots)
                    : launch_layout<float>(d, p, tile, s, sumsq_slots);
}

}  // namespace lsam
