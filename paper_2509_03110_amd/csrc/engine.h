// Internal declarations shared by the host engine and the kernel launchers.
// Nothing here is part of the public boundary (include/lsam.h).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/lsam.h"
#include "b32s.h"
#include "langevin.h"

namespace lsam {

constexpr int kMaxK = LSAM_MAX_REPLICAS;

// Small per-replica tables handed to kernels by value.
struct ReplicaScalars {
  float v[kMaxK];
};
struct DueList {
  int32_t n;
  int32_t idx[kMaxK];
};

// Message that lsam_last_error() returns on the calling thread (copied).
void set_last_error(const char* msg);

// One coordinate of the sampler step (Algorithm 2, asynchronous sampling step, driven by
// momentum SGD): G = g + lam (x - y); v <- mu v + G; x <- x - lr (G + mu v) [Nesterov] or
// x - lr v [heavy ball], plus the Langevin term xi (0 without noise); S <- S + x.  The one
// definition both the streaming kernel and the fused GEMM epilogue use, so that they round alike.
__device__ __forceinline__ void sampler_step(float g, float y, float lam, float lr, float mu,
                                             int nesterov, float xi, float& x, float& v, float& S) {
  const float G = g + lam * (x - y);
  const float vn = mu * v + G;
  const float xn = (nesterov ? x - lr * (G + mu * vn) : x - lr * vn) + xi;
  v = vn;
  x = xn;
  S += xn;
}

// One coordinate of the ascent step x~ = x + scale g, scale = rho / (||g|| + gamma) (Formulation,
// first-order solution of the inner maximisation); shared by the streaming kernel and the
// GEMM epilogue for the same reason.
__device__ __forceinline__ float ascent_point(float x, float scale, float g) {
  return __builtin_fmaf(scale, g, x);
}

// ---- streaming kernels (update path) ---------------------------------------------------

// Sum of squares, pass 1: per (replica, block) partial sums in double.
// g: [K] rows of `n` floats with row stride `g_stride`; partials: [K, nblk] doubles.
void launch_sumsq_partials(const float* g, int64_t g_stride, int64_t n, int K, double* partials,
                           int nblk, hipStream_t s);
// Inner product of K pairs of matrices G1, G2 (each `n` floats, replica stride `stride`, both
// multiples of 4, 16-byte aligned): partials[k * pstride + j] for j < the returned count (<= 64).
// G1 (G2) is the sum of pieces1 (pieces2) >= 1 partial matrices lying piece_stride elements apart.
int launch_gram_dot(const float* G1, const float* G2, int64_t stride, int64_t n, int K, int pieces1,
                    int pieces2, int64_t piece_stride, double* partials, int64_t pstride, hipStream_t s);
// Pass 2: norms[k] = sqrt(sum_{b<nblk} partials[k * partials_stride + b]); scale[k] = rho / (norm + gamma).
// If loss_rows != nullptr also reduces loss_rows [K,B] to loss_out[k] = mean (both passes of
// the tree are fixed-order, so the result is run-to-run deterministic).
// `restart` (may be null): the per-replica marks described at launch_center; this kernel, which
// runs once per step before anything touches the iterate sums, counts every mark down by one.
void launch_norm_finish(const double* partials, int nblk, int64_t partials_stride, int K, float rho, float gamma,
                        float* norms, float* scale, const float* loss_rows, int B,
                        float* loss_out, hipStream_t s, int32_t* restart = nullptr);
// x~ = x + scale[k] * g.  Writes fp32 (xt_f32), or, if xt_bf16 is non-null, the bf16 operand
// copy of the weight matrices in the blocked layout described by `map` (replica stride
// `shadow_stride` elements).
void launch_perturb(const float* x, const float* g, int64_t g_stride, const float* scale,
                    float* xt_f32, uint16_t* xt_bf16, const ShadowMap* map, int64_t shadow_stride,
                    int64_t stride, int64_t n, int K, hipStream_t s);
// Descent + coupling for all K replicas, y read once per index:
//   G = g + lam[k] (x - y); v = mu v + G; x -= lr (G + mu v) [nesterov] | lr v; S += x.
// Also refreshes the bf16 operand copy of the weight matrices if `shadow` is non-null, and adds
// the Langevin noise described by `noise` (null: none) to the new x.  A replica whose mark in
// `restart` (may be null) is 1 starts its sum afresh: S = x, without reading S.
void launch_descent(float* x, const float* g, int64_t g_stride, float* v, float* S,
                    const float* y, uint16_t* shadow, const ShadowMap* map, int64_t shadow_stride,
                    int64_t stride, int64_t n, int K, const ReplicaScalars& lam, float lr, float mu,
                    int nesterov, const NoiseMap* noise, hipStream_t s, const int32_t* restart = nullptr);
// dst[c * dst_stride + i] = (1/K) sum_k src[k * src_stride + i] for c < copies, i < n; the K
// terms are added in replica order.  dst may be src (each index is read in full before it is
// written).
void launch_grad_mean(const float* src, int64_t src_stride, float* dst, int64_t dst_stride,
                      int64_t n, int K, int copies, hipStream_t s);
// Center update over the due replicas (Algorithm 2, synchronous optimization step).  The sums of
// the due replicas start again from zero afterwards.  Without `restart` the kernel writes the
// zeros.  With it (K words of device memory, zero at first) it writes none: it sets the mark of
// every due replica to 2, which means "this sum reads as zero, its memory is stale"; the next
// step's launch_norm_finish makes that a 1, which tells that step's sampler kernels to start the
// sum from x alone instead of reading it, and the step after makes it 0 again.  All of it is
// data on the device, so a captured step replays correctly.  Saves writing and reading back
// 4 bytes per parameter of every replica served.
void launch_center(float* S, float* y, float* gprev, int64_t stride, int64_t n,
                   const DueList& due, float inv_m, float beta, float lr_center, int has_prev,
                   hipStream_t s, int32_t* restart = nullptr);
// dst[k, :] = src[:] for k < K (fp32).
void launch_broadcast(const float* src, float* dst, int64_t stride, int64_t n, int K, hipStream_t s);
// Rebuilds the bf16 operand copy of K replicas from their fp32 parameters.
void launch_shadow_refresh(const float* x, uint16_t* shadow, const ShadowMap& map, int64_t stride,
                           int64_t shadow_stride, int64_t n, int K, hipStream_t s);
// Row-major bf16 [K][rows][cols] -> blocked layout, one matrix per replica (dst pre-zeroed
// padding is left untouched).
void launch_rowmajor_to_b32s(const uint16_t* src, uint16_t* dst, int rows, int cols, int K,
                             hipStream_t s);
void launch_fill_zero(void* p, size_t bytes, hipStream_t s);
// Row-padded copy: dst[r, 0:cols] = src[r, 0:cols], rows of `elem` bytes-sized elements.
void launch_pad_rows(const void* src, void* dst, int64_t rows, int cols, int ld_dst, int elem,
                     hipStream_t s);

// ---- model kernels ------------------------------------------------------------------------

enum GemmEpilogue { EPI_BIAS = 0, EPI_BIAS_RELU = 1, EPI_MASK = 2, EPI_PLAIN = 3 };

// C[k][m, n] = sum_kk A(k; m, kk) * B(k; n, kk), batched over replicas k.
// An operand is "k-major" when kk is its contiguous index (row pitch ld along m resp. n),
// otherwise "m-major" (kk selects the row, m resp. n is contiguous).
struct GemmDesc {
  const void* A; int64_t strideA; int ldA; int a_kmajor;
  const void* B; int64_t strideB; int ldB; int b_kmajor;
  void* C; int64_t strideC; int ldC;
  int M, N, Kd, batch;
  int in_bf16;        // operands bf16 (else fp32)
  int out_bf16;       // output bf16 (else fp32)
  int epilogue;       // GemmEpilogue
  const float* bias; int64_t strideBias;          // EPI_BIAS*: bias[n]
  const float* bias_dir; const float* bias_scale; // if set: bias[n] + bias_scale[k] * bias_dir[n]
  const void* mask; int64_t strideMask; int ldMask; // EPI_MASK: keep where mask[m,n] > 0 (operand dtype)
  float* splitk_ws; size_t splitk_bytes;            // scratch for split-K partial sums (may be null)
  // bf16 tensors in the blocked layout (b32s.h): column blocks of the stored A, B, bf16 C, mask;
  // strideA/B/C/Mask then count elements of one replica's stored matrix and ld* are unused
  int b32s; int cbA, cbB, cbC, cbMask;
  // If set (fp32 results only): every workgroup that writes results also writes the sum of
  // their squares, in double, to sumsq[k * sumsq_stride + slot], slot = 0 .. slots-1 inside a
  // replica; `slots` comes back through launch_gemm.  Fixed summation order.
  double* sumsq; int64_t sumsq_stride;
  // fp32 only.  unfold = 1: A is not stored as [M][Kd]; it is the unfolded image of a 3x3
  // convolution (stride 1, zero rim 1) read straight from the image A points to, [M pixels]
  // [unfold_C] with M a multiple of unfold_H * unfold_W, Kd = 9 * unfold_C, both operands
  // k-major.  unfold = 2: the same for B as an m-major operand: B points to the image
  // [Kd pixels][unfold_C], N = 9 * unfold_C, both operands m-major.  unfold_C must be a
  // multiple of 32; ldA resp. ldB is then ignored apart from the alignment checks.
  int unfold, unfold_C, unfold_H, unfold_W;
  // fp32 operands only: round both operands to bfloat16 on their way into the matrix unit
  // (v_mfma_f32_32x32x16_bf16, fp32 accumulate); memory traffic and results stay fp32.
  int bf16_math;
  // If set (bf16 operands, fp32 result, EPI_PLAIN): the result, a weight gradient at the
  // perturbed point, is not stored.  The epilogue takes the sampler step on it instead
  // (Algorithm 2, asynchronous sampling step, with Nesterov or heavy-ball momentum), element
  // (m, n) of replica k living at offset k * strideC + m * ldC + n of x, v and S and at
  // m * ldC + n of y:  G = C + lam[k] (x - y);  v = mu v + G;  x -= lr (G + mu v)  [or lr v];
  // S += x;  and bf16(x) goes to the blocked operand copy `shadow` (replica stride
  // shadow_stride elements, cbShadow column blocks).  C is ignored.
  const struct SamplerFusion* fuse;
  // If set (same kind of launch, a weight gradient of the first pass recomputed once its norm
  // is known): the result is not stored either; the epilogue writes the operand copy of the
  // perturbed weights, bf16(x + scale[k] * C), x addressed like the result.
  const struct AscentFusion* ascend;
  // If set (same kind of launch, `sumsq` given): only the sums of squares are written.
  int sumsq_only;
  // bf16 operands in the blocked layout, plain fp32 result, none of the options above: with
  // ksplit > 1 the contraction is cut into ksplit pieces of whole 32-deep steps, each taken by
  // workgroups of its own, and piece j writes its partial result at C + j * split_stride
  // (elements, beside the replica stride); the caller adds the pieces up in a fixed order.
  int ksplit; int64_t split_stride;
};
struct AscentFusion {
  const float* x; const float* scale;
  uint16_t* shadow; int64_t shadow_stride; int cbShadow;
};
struct SamplerFusion {
  float* x; float* v; float* S; const float* y;
  uint16_t* shadow; int64_t shadow_stride; int cbShadow;
  ReplicaScalars lam;
  float lr, mu;
  int nesterov;
  const int32_t* restart;     // marks of launch_center (may be null)
};
// 0 ok, <0 unsupported shape; *sumsq_slots (if non-null) = slots written per replica
int launch_gemm(const GemmDesc& d, hipStream_t s, int* sumsq_slots = nullptr);
// Upper bound of the slots any launch of an [M, N] result can use.
int gemm_sumsq_capacity(int M, int N);
size_t gemm_splitk_bytes(const GemmDesc& d);          // scratch this GEMM would like (0: none)
// bf16 fast path (direct-to-LDS ring); returns 1 when the shape is left to the generic kernel.
int launch_gemm_bf16(const GemmDesc& d, int tile_override, hipStream_t s, int* sumsq_slots);

// Softmax cross-entropy, forward and backward.  logits [K,B,ld] fp32; labels [K,B];
// dz = (softmax - onehot)/B: fp32 [K,B,ld_dz] row-major with zeros in the padded columns, or
// (dz_bf16) bf16 in the blocked layout, ld_dz then being one replica's stored size in elements;
// loss_rows [K,B] = lse - logit[label] (may be null).
void launch_softmax_ce(const float* logits, int ld, const int32_t* labels, void* dz, int64_t ld_dz,
                       int dz_bf16, float* loss_rows, int K, int B, int C, hipStream_t s);
// db[k][n] = sum_b dz[k][b][n]; dz as written by the kernels above (ld: row pitch, or one
// replica's stored size for the blocked bf16 layout).
// If sumsq is non-null, workgroup j of replica k also writes the sum of squares of its 64
// results to sumsq[k * sumsq_stride + j]; returns the number of such slots per replica.
int launch_bias_grad(const void* dz, int64_t ld, int dz_bf16, float* db, int64_t strideDb, int K,
                     int B, int N, double* sumsq, int64_t sumsq_stride, hipStream_t s);

// Narrow classifier head in fp32 (head_fits: few classes, an input row that fits LDS, a
// moderate batch): forward of the last layer, loss, dZ and the masked dX in one kernel (A: the
// layer's input [K,B,ld], a ReLU output, ld = `in` rounded up to 8; W, bias: the layer's
// parameters inside each replica, replica stride strideW, row pitch ld; dz [K,B,ld_dz] gets
// the padded dZ; dA [K,B,ld], if non-null, dZ W where A > 0; returns <0 if the launch could
// not be set up), and its weight and bias gradient in another (dW, db inside each replica's
// gradient, stride strideG; returns the sum-of-squares slots written per replica, which is
// head_sumsq_slots(in)).
bool head_fits(int B, int C, int in);
int head_sumsq_slots(int in);
int launch_head_forward_backward(const float* A, const float* W, const float* bias, int64_t strideW,
                                 const int32_t* labels, float* dz, int ld_dz, float* loss_rows,
                                 float* dA, int K, int B, int C, int in, hipStream_t s);
int launch_head_weight_grad(const float* dz, int ld_dz, const float* A, int ldA, float* dW, int ldw,
                            float* db, int64_t strideG, int K, int B, int C, int in, double* sumsq,
                            int64_t sumsq_stride, hipStream_t s);

// 3x3 convolution support (fp32, tensors [K][B][H][W][C], C contiguous).  All return 0, or -1
// when the shape does not fit the kernel (pitches and channel counts that are not multiples
// of 4 where stated).
// col[k][(b,i,j)][(u,v,c)] = X[k][b][i+u-1][j+v-1][c], zero outside the image and in the
// padding columns 9C..ld-1 (ld % 4 == 0; any C).
// `stride` 1 or 2: the image is [stride H][stride W][C] and col row (b,i,j) holds the window
// around pixel (stride i, stride j); H x W is the convolution's output.
int launch_unfold3x3(const float* X, int64_t strideX, float* col, int64_t strideCol, int ld, int K,
                     int B, int H, int W, int C, int stride, hipStream_t s);
// dX[k][b][i][j][c] = sum_{u,v} dcol[k][(b,i-u+1,j-v+1)][(u,v,c)], taps added in (u,v) order,
// set to zero where mask (same shape as dX, may be null) is not positive.  C % 4 == 0.
int launch_fold3x3(const float* dcol, int64_t strideCol, int ld, float* dX, const float* mask,
                   int64_t strideX, int K, int B, int H, int W, int C, int stride, hipStream_t s);
// A first convolution layer with C = 1..3 input channels and a multiple of 32 output channels
// (first_conv_fits) has kernels of its own that gather the image straight into the MFMA
// operands.  Forward: out[k][p][o] = b[o] + conv, rectified if `relu`, parameters taken from
// params + k * strideParams at w_off (row pitch ldw) and b_off.  Weight gradient: dW and db
// into grad + k * strideParams at the same offsets, through `partial`
// ([K][first_conv_chunks(rows)][Cout][32] floats of scratch), plus, if sumsq is non-null, the
// sums of their squares in sumsq[k * sumsq_stride + slot]; returns the slots written per
// replica (Cout / 2), or -1.  `round`: both operands of every product are rounded to bfloat16
// first.  `skip_bias`: the weight-gradient kernels leave db alone (with rounded operands they
// would sum rounded values, the caller then takes the column sums of dout instead; below a
// batch normalisation the bias gradient is zero).
bool first_conv_fits(int C, int Cout, int64_t rows);
int first_conv_chunks(int64_t rows);
int launch_first_conv_forward(const float* X, const float* params, int64_t strideParams, int64_t w_off,
                              int64_t b_off, int ldw, float* out, int relu, int round, int K,
                              int64_t rows, int H, int W, int C, int Cout, hipStream_t s);
int launch_first_conv_wgrad(const float* X, const float* dout, float* partial, float* grad,
                            int64_t strideParams, int64_t w_off, int64_t b_off, int ldw, int round,
                            int skip_bias, int K, int64_t rows, int H, int W, int C, int Cout,
                            double* sumsq, int64_t sumsq_stride, hipStream_t s);
// Training-mode batch normalisation of K matrices Z [rows][C] (C % 4 == 0, C <= 1024), per
// replica and column over the rows.  Forward: stats[k][0][c] = mean, stats[k][1][c] =
// 1/sqrt(biased variance + eps); out = relu(gamma Xh + beta), Xh = (Z - mean) stats[1], gamma
// and beta read from params + k * strideParams at gam_off / bet_off.  `scratch`: 2 * K *
// bn_chunks(rows, C, K) * C floats.  Backward: launch_bn_backward_partials leaves chunk sums
// part[k][chunk][0..C) = sum dY Xh and [C..2C) = sum dY (returns the chunk count; launch_bias_grad
// over them gives dgamma and dbeta); launch_bn_backward_apply then writes
// dZ = gamma stats[1] (dY - dbeta/rows - Xh dgamma/rows) to `dZ`, which may be dY itself or Z,
// dgamma and dbeta read from grad + k * strideParams at the same offsets.  -1: shape not supported.
// Shortcut of a residual block (He et al., CIFAR variant, parameter-free): the block input
// src [K][B][step H][step W][Cs] (replica stride `stride` floats) enters the block output
// [B][H][W][C] as src[b][step i][step j][c] for c < Cs and 0 for the channels beyond.  Cs % 4 == 0.
// A projection shortcut instead (that paper's 1x1 convolution with batch normalisation): `pz`
// [K][rows][C] is the 1x1 convolution's output, `pstats` its statistics (launch_bn_stats), and
// gamma_p, beta_p sit at pgam_off, pbet_off of each replica's parameters; pz null: no projection.
struct ShortcutDesc {
  const float* src; int64_t stride;
  int H, W, Cs, step;
  const float* pz = nullptr; const float* pstats = nullptr;
  int64_t pgam_off = 0, pbet_off = 0;
};
// stats[k] = (mean, 1/sqrt(var + eps)) per channel of Z [K][rows][C]; scratch as for launch_bn_forward.
int launch_bn_stats(const float* Z, float* scratch, float* stats, int K, int64_t rows, int C, float eps,
                    hipStream_t s);
// dst[i] += src[i] for i < n (n % 4 == 0; both 16-byte aligned, not overlapping).
int launch_add_into(float* dst, const float* src, int64_t n, hipStream_t s);
// dst[img][i][j][c] = src[img][2 i][2 j][c] for `images` images [2H][2W][C] (C % 4 == 0).
int launch_subsample2(const float* src, float* dst, int64_t images, int H, int W, int C, hipStream_t s);
int bn_chunks(int64_t rows, int C, int K);
// `shortcut` (may be null): added to the normalised output before the ReLU.
int launch_bn_forward(const float* Z, float* scratch, float* stats, const float* params,
                      int64_t strideParams, int64_t gam_off, int64_t bet_off, float* out, int K,
                      int64_t rows, int C, float eps, const ShortcutDesc* shortcut, hipStream_t s);
// dIn (shape of d.src) += the gradient dY [K][rows][C] of the block output, through the shortcut,
// kept only where mask (shape of dIn, the ReLU output the block read; may be null) is positive.
int launch_shortcut_backward(const float* dY, float* dIn, const float* mask, const ShortcutDesc& d, int K,
                             int64_t rows, int C, hipStream_t s);
// Global average pooling over `images` images [HW][C] into rows of pitch ldp, and its backward
// pass fused with the ReLU mask of the image (mask may be null).
int launch_avgpool(const float* A, float* P, int64_t images, int HW, int C, int ldp, hipStream_t s);
int launch_avgpool_backward(const float* dP, const float* mask, float* dA, int64_t images, int HW, int C,
                            int ldp, hipStream_t s);
int launch_bn_backward_partials(const float* Z, const float* dY, const float* stats, float* part, int K,
                                int64_t rows, int C, hipStream_t s);
void launch_bn_backward_apply(const float* Z, const float* dY, float* dZ, const float* stats,
                              const float* params, const float* grad, int64_t strideParams,
                              int64_t gam_off, int64_t bet_off, int K, int64_t rows, int C, hipStream_t s);
// Wt[k][c][(u,v,o)] = W[k][o][(2-u,2-v,c)] for K filter banks W [Cout][3][3][Cin] (row pitch ldw,
// replica stride strideW); Wt is dense, [K][Cin][9 Cout].  Cout must be a multiple of 32.
void launch_flip_filters(const float* W, int64_t strideW, int ldw, float* Wt, int K, int Cout, int Cin,
                         hipStream_t s);
// Column sums of K contiguous [rows][N] matrices, first stage: partial[k][chunk][n] = sum of
// the rows of chunk `chunk` (colsum_chunks(rows, N, K) chunks of equal height, the last one ragged);
// returns the chunk count, -1 if N is not a multiple of 4 in 4..1024.  launch_bias_grad over
// the partials finishes the sum.
int colsum_chunks(int64_t rows, int N, int K);
int launch_colsum_partials(const float* A, int64_t rows, int N, int K, float* partial, hipStream_t s);
// 2x2/stride-2 max-pool over `images` contiguous [H][W][C] images, and the backward pass of
// ReLU-then-pool: dA = dP at the first maximum of each window if it is positive, else 0
// (A: the ReLU output that was pooled).  C % 4 == 0, H and W even.
int launch_maxpool2(const float* A, float* P, int64_t images, int H, int W, int C, hipStream_t s);
int launch_maxpool2_backward(const float* A, const float* dP, float* dA, int64_t images, int H,
                             int W, int C, hipStream_t s);

// Measured ceilings: device copy (GB/s, read + written) between the halves of `scratch`, and
// MFMA-only loops (TFLOP/s, bf16 32x32x16 and fp32 32x32x2).  Blocks until done; 0 or -1.
int probe_peaks(void* scratch, size_t bytes, hipStream_t s, double* copy_gbs, double* bf16_tflops,
                double* f32_tflops);

}  // namespace lsam
