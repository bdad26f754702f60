// Host engine behind include/lsam.h: configuration checks, workspace carve-up, the integer
// communication schedule, and the kernel sequence of one LSAM step / one center update.
#include <algorithm>
#include <climits>
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <new>
#include <string>
#include <vector>

#include "engine.h"

namespace lsam {
namespace {

thread_local std::string g_err;

int fail(int code, const char* fmt, ...) {
  char buf[512];
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(buf, sizeof buf, fmt, ap);
  va_end(ap);
  g_err = buf;
  return code;
}

#define HIP_TRY(expr)                                                                   \
  do {                                                                                  \
    hipError_t e_ = (expr);                                                             \
    if (e_ != hipSuccess) return fail(LSAM_EHIP, "%s: %s", #expr, hipGetErrorString(e_)); \
  } while (0)

inline int64_t round_up(int64_t v, int64_t a) { return (v + a - 1) / a * a; }

// ---- communication schedule (integers only) -------------------------------------------------
// Period generator: s_{j+1} = A s_j + C mod 2^64, draw_j = (s_{j+1} >> 33) mod range + min.
// Replica i is due when its local count reaches its period: the trigger of Algorithm 2's
// synchronous optimization step (total local iterations reaching a multiple of n tau), taken
// per replica so that periods may differ; with equal periods every replica is due at the same
// tick and the two coincide.
class Schedule {
 public:
  void init(const lsam_config& c) {
    K_ = c.K;
    lo_ = c.tau_min;
    hi_ = c.tau_max;
    redraw_ = c.sched_mode == LSAM_SCHED_REDRAW;
    state_ = c.sched_seed;
    explicit_ = c.tau != nullptr;
    tau_.resize(K_);
    count_.assign(K_, 0);
    t_y_ = 0;
    for (int i = 0; i < K_; ++i) tau_[i] = explicit_ ? c.tau[i] : draw();
  }
  int32_t draw() {
    state_ = state_ * 6364136223846793005ULL + 1442695040888963407ULL;
    const uint64_t range = (uint64_t)(hi_ - lo_ + 1);
    return (int32_t)((state_ >> 33) % range) + lo_;
  }
  void tick() {
    for (int i = 0; i < K_; ++i) ++count_[i];
  }
  DueList due() const {
    DueList d;
    d.n = 0;
    for (int i = 0; i < K_; ++i)
      if (count_[i] >= tau_[i]) d.idx[d.n++] = i;
    return d;
  }
  int64_t samples(const DueList& d) const {
    int64_t m = 0;
    for (int j = 0; j < d.n; ++j) m += count_[d.idx[j]];
    return m;
  }
  void served(const DueList& d) {
    for (int j = 0; j < d.n; ++j) {
      count_[d.idx[j]] = 0;
      if (redraw_ && !explicit_) tau_[d.idx[j]] = draw();
    }
    ++t_y_;
  }
  const std::vector<int32_t>& tau() const { return tau_; }
  const std::vector<int32_t>& count() const { return count_; }
  int64_t t_y() const { return t_y_; }
  uint64_t generator_state() const { return state_; }
  // Overwrites counts, periods in force, the generator state and the sync count (resume).
  bool restore(const int64_t* count, const int64_t* tau, uint64_t state, int64_t t_y) {
    if (t_y < 0) return false;
    for (int i = 0; i < K_; ++i)
      if (count[i] < 0 || count[i] > INT32_MAX || tau[i] < 1 || tau[i] > INT32_MAX) return false;
    for (int i = 0; i < K_; ++i) {
      count_[i] = (int32_t)count[i];
      tau_[i] = (int32_t)tau[i];
    }
    state_ = state;
    t_y_ = t_y;
    return true;
  }

 private:
  int K_ = 0, lo_ = 1, hi_ = 1;
  bool redraw_ = false, explicit_ = false;
  uint64_t state_ = 0;
  std::vector<int32_t> tau_, count_;
  int64_t t_y_ = 0;
};

// ---- layout -----------------------------------------------------------------------------------
struct Layer {
  int in, out;          // true extents
  int ldw;              // row pitch of W in the padded layout (floats)
  int64_t w_off, b_off; // offsets inside one replica of the padded layout (floats)
  int64_t w_flat, b_flat; // offsets inside the public flat layout
  bool bn = false;        // batch-normalised convolution: gamma and beta follow the bias
  int64_t gam_off = 0, bet_off = 0, gam_flat = 0, bet_flat = 0;
  // projection shortcut closed by this convolution: W_p [out][proj_in] (row pitch proj_in, a
  // multiple of 8), b_p, gamma_p, beta_p follow the layer's own parameters
  bool proj = false;
  int proj_in = 0;
  int64_t pw_off = 0, pb_off = 0, pgam_off = 0, pbet_off = 0;
};

// One parameter group as the copies between the flat and the padded layout and the noise
// generator see it: `rows` rows of `cols` values, row pitch `ld` in the padded layout.
struct Piece {
  int64_t off, flat;
  int rows, cols, ld;
  int code;               // 8 * layer + {0 W, 1 b, 2 gamma, 3 beta, 4..7 the projection's four}
};

// One 3x3 convolution layer: image [H][W][Cin] -> [H][W][Cout] (-> [H/2][W/2][Cout] if pooled).
struct ConvLayer {
  int H, W, Cin, Cout, pool;   // H x W: the convolution's output image (before the pool)
  int stride;          // 1 or 2: the layer reads an image of [stride H][stride W][Cin]
  bool skip;           // closes a residual block: the input of the layer below is added before the ReLU
  int skip_C, skip_step;   // channels of that block input; 2 if the block halved the image, else 1
  bool proj;           // that shortcut is a projection (1x1 convolution + batch normalisation)
  size_t psub, pz, pstats; // its input pixels [K][rows][skip_C] (later: their gradient), its
                           // convolution output [K][rows][Cout] (later: that output's gradient), its statistics
  int64_t rows;        // B H W: rows of the unfolded image and of the layer's output
  int ldc;             // pitch of the unfolded image, 9 Cin rounded up to 8
  // The GEMM kernels can read an unfolded image straight from the image when its channel
  // count is a multiple of 32: `direct_in` for the layer's input (forward and dW), `direct_dx`
  // for its output gradient (dX, with the mirrored filters `wt`).  Otherwise the unfolded
  // image (`col`) resp. its gradient (the shared `dcol`) is stored.
  // `first`: layer 0 with 1..3 input channels runs its forward pass and its weight gradient
  // in kernels of their own (no unfolded image at all).
  bool direct_in, direct_dx, first;
  size_t first_partial;   // scratch of the first layer's weight gradient
  bool bn;                // batch-normalised: `z` keeps the convolution's output, `stats` the
  size_t z, stats;        // per-channel mean and 1/sqrt(var + eps) of each replica
  size_t col, out, pooled, dout, dpooled, wt;   // workspace offsets ([K] contiguous replicas each)
};

struct Layout {
  int K = 0, L = 0, B = 0;
  int n_conv = 0;              // layers 0..n_conv-1 are convolutions
  bool preact = false;         // residual blocks sum un-normalised convolution outputs (wide residual networks)
  std::vector<ConvLayer> conv;
  size_t dcol = 0;             // gradient of an unfolded image (largest layer that needs one)
  size_t gram1 = 0, gram2 = 0; // bf16 dense model: Gram matrices [K][B][ldg] of a layer's dZ and of its input
  size_t restart = 0;         // K marks: which iterate sums read as zero / start afresh (launch_center)
  int ldg = 0;
  int gap_hw = 0;              // > 0: global average pooling over that many positions feeds the dense layers
  size_t gap_out = 0, gap_grad = 0;   // [K][B][ld] pooled vector and its gradient
  size_t colsum = 0;           // first-stage column sums of the bias gradients
  bool bf16 = false, raw = false;
  bool bf16_math = false;      // convolutional model with bf16 matrix products on fp32 tensors
  int64_t d = 0, d_pad = 0;
  std::vector<Layer> layers;
  std::vector<Piece> pieces; // every parameter group, in the order of the flat layout
  size_t noise_segs = 0;     // device copy of the noise generator's table (Langevin sampler only)
  std::vector<int> ld;       // activation pitches ld[0..L]
  bool need_a0 = false;
  int nblk = 1;
  // byte offsets into the workspace
  size_t gmean = 0;   // raw-vector mode, data-parallel baseline: the averaged gradient [d_pad]
  size_t x = 0, g = 0, v = 0, S = 0, xt = 0, y = 0, gprev = 0, partials = 0, norms = 0, scale = 0,
         loss_rows = 0, loss = 0, logits = 0, a0 = 0, splitk = 0, splitk_bytes = 0, total = 0;
  std::vector<size_t> act, dz;  // act[l] for l = 1..L-1, dz[l] for l = 1..L (index l)
  // bf16 mode: every bf16 tensor is stored in the blocked layout (b32s.h)
  std::vector<int64_t> shadow_off;   // offset of W_l's operand copy inside a replica's copy
  int64_t shadow_stride = 0;         // elements of one replica's operand copy
  ShadowMap map{};
  size_t es() const { return bf16 ? 2 : 4; }
  // elements of one replica's stored [B][dims] activation-like matrix
  int64_t act_elems(int width, int pitch) const {
    return bf16 ? b32s_size(B, width) : (int64_t)B * pitch;
  }
};

int check_config(const lsam_config* c) {
  if (!c) return fail(LSAM_EINVAL, "config is NULL");
  if (c->K < 1 || c->K > LSAM_MAX_REPLICAS)
    return fail(LSAM_EINVAL, "K=%d outside 1..%d", c->K, LSAM_MAX_REPLICAS);
  if (c->n_layers < 0 || c->n_layers > LSAM_MAX_LAYERS)
    return fail(LSAM_EINVAL, "n_layers=%d outside 0..%d", c->n_layers, LSAM_MAX_LAYERS);
  if (c->n_layers == 0) {
    if (c->d_raw < 1) return fail(LSAM_EINVAL, "raw-vector mode needs d_raw >= 1");
  } else {
    if (!c->dims) return fail(LSAM_EINVAL, "dims is NULL");
    for (int l = 0; l <= c->n_layers; ++l)
      if (c->dims[l] < 1) return fail(LSAM_EINVAL, "dims[%d]=%d must be >= 1", l, c->dims[l]);
    if (c->batch < 1) return fail(LSAM_EINVAL, "batch must be >= 1");
    if ((int64_t)c->K * c->batch > (1 << 24)) return fail(LSAM_EINVAL, "K*batch too large");
    if (c->gemm_dtype != LSAM_GEMM_FP32 && c->gemm_dtype != LSAM_GEMM_BF16)
      return fail(LSAM_EINVAL, "gemm_dtype must be 0 (fp32) or 1 (bf16)");
    if (c->n_conv < 0 || c->n_conv >= c->n_layers)
      return fail(LSAM_EINVAL, "n_conv=%d must leave at least one dense layer of %d", c->n_conv,
                  c->n_layers);
    if (c->n_conv == 0 && c->bn_mask) return fail(LSAM_EINVAL, "bn_mask needs convolution layers");
    if (c->n_conv == 0 && (c->stride_mask || c->skip_mask || c->proj_mask || c->global_avg_pool || c->preact))
      return fail(LSAM_EINVAL, "stride_mask, skip_mask, proj_mask, global_avg_pool and preact need convolution layers");
    if (c->n_conv > 0) {
      if (c->img_h < 1 || c->img_w < 1) return fail(LSAM_EINVAL, "img_h, img_w must be >= 1");
      if (c->bn_mask >> c->n_conv) return fail(LSAM_EINVAL, "bn_mask names a layer that is no convolution");
      if (c->bn_mask && !(c->bn_eps > 0.f)) return fail(LSAM_EINVAL, "bn_eps must be > 0");
      if ((c->stride_mask >> c->n_conv) || (c->skip_mask >> c->n_conv) || (c->pool_mask >> c->n_conv))
        return fail(LSAM_EINVAL, "stride_mask, skip_mask or pool_mask names a layer that is no convolution");
      if (c->proj_mask & ~c->skip_mask)
        return fail(LSAM_EINVAL, "proj_mask names a layer that closes no residual block");
      if (c->global_avg_pool != 0 && c->global_avg_pool != 1)
        return fail(LSAM_EINVAL, "global_avg_pool must be 0 or 1");
      if (c->preact != 0 && c->preact != 1) return fail(LSAM_EINVAL, "preact must be 0 or 1");
      if (c->preact && c->bn_mask != ((1ull << c->n_conv) - 1))
        return fail(LSAM_EINVAL, "pre-activation blocks need every convolution batch-normalised");
      int64_t h = c->img_h, w = c->img_w;
      int64_t in_h[LSAM_MAX_LAYERS + 1], in_w[LSAM_MAX_LAYERS + 1];   // image each convolution reads
      for (int l = 0; l < c->n_conv; ++l) {
        in_h[l] = h; in_w[l] = w;
        if (c->dims[l + 1] % 8)
          return fail(LSAM_EINVAL, "dims[%d]=%d: convolution outputs must be multiples of 8", l + 1,
                      c->dims[l + 1]);
        if ((c->stride_mask >> l) & 1u) {
          if (h % 2 || w % 2)
            return fail(LSAM_EINVAL, "convolution %d: stride 2 needs even image sides (%lldx%lld)", l,
                        (long long)h, (long long)w);
          h /= 2;
          w /= 2;
        }
        if ((c->skip_mask >> l) & 1u) {
          if (l < 2) return fail(LSAM_EINVAL, "convolution %d: a residual block needs two convolutions below its closing one", l);
          if (!((c->bn_mask >> l) & 1u))
            return fail(LSAM_EINVAL, "convolution %d: the closing convolution of a residual block must be batch-normalised", l);
          if (((c->pool_mask >> (l - 1)) & 1u) || ((c->pool_mask >> (l - 2)) & 1u))
            return fail(LSAM_EINVAL, "convolution %d: no pool may sit inside a residual block or in front of it", l);
          const int64_t sh = in_h[l - 1], sw = in_w[l - 1];
          const bool proj = ((c->proj_mask >> l) & 1u) != 0;
          // (a pre-activation block without projection adds two sums of the same shape)
          if (!((sh == h && sw == w) || (sh == 2 * h && sw == 2 * w)) ||
              (!proj && c->dims[l - 1] > c->dims[l + 1]) || c->dims[l - 1] % (proj ? 8 : 4) ||
              (c->preact && !proj && (sh != h || sw != w || c->dims[l - 1] != c->dims[l + 1])))
            return fail(LSAM_EINVAL, "convolution %d: the block input (%lldx%lldx%d) does not fit the block output (%lldx%lldx%d)",
                        l, (long long)sh, (long long)sw, c->dims[l - 1], (long long)h, (long long)w, c->dims[l + 1]);
        }
        // one replica's unfolded image is a GEMM operand addressed with 32-bit byte offsets
        const int64_t widest = std::max<int64_t>(round_up(9 * (int64_t)c->dims[l], 8), c->dims[l + 1]);
        if ((int64_t)c->batch * h * w * widest * 4 >= 0x7FFFFFF0LL)
          return fail(LSAM_EINVAL, "convolution %d: batch * image * channels too large", l);
        if ((c->pool_mask >> l) & 1u) {
          if (h % 2 || w % 2)
            return fail(LSAM_EINVAL, "convolution %d: pooling needs even image sides (%lldx%lld)", l,
                        (long long)h, (long long)w);
          h /= 2;
          w /= 2;
        }
      }
      if (!c->global_avg_pool && h * w * c->dims[c->n_conv] > (1 << 24))
        return fail(LSAM_EINVAL, "flattened image too wide for the dense layers");
    }
  }
  if (!(c->rho >= 0.f) || !(c->gamma >= 0.f)) return fail(LSAM_EINVAL, "rho, gamma must be >= 0");
  if (!(c->lr > 0.f) && c->lambda_abs < 0.f)
    return fail(LSAM_EINVAL, "lr must be > 0 when lambda is derived as lambda0/(lr*tau)");
  if (!(c->lr >= 0.f)) return fail(LSAM_EINVAL, "lr must be >= 0");
  if (!(c->momentum >= 0.f && c->momentum < 1.f))
    return fail(LSAM_EINVAL, "momentum must be in [0,1)");
  if (!std::isfinite(c->beta) || !std::isfinite(c->lr_center) || !std::isfinite(c->lambda0))
    return fail(LSAM_EINVAL, "beta, lr_center, lambda0 must be finite");
  if (c->tau) {
    for (int i = 0; i < c->K; ++i)
      if (c->tau[i] < 1) return fail(LSAM_EINVAL, "tau[%d]=%d must be >= 1", i, c->tau[i]);
  } else {
    if (c->tau_min < 1 || c->tau_max < c->tau_min)
      return fail(LSAM_EINVAL, "need 1 <= tau_min <= tau_max");
  }
  if (c->sched_mode != LSAM_SCHED_FIXED && c->sched_mode != LSAM_SCHED_REDRAW)
    return fail(LSAM_EINVAL, "sched_mode must be 0 or 1");
  if (c->algorithm != LSAM_ALG_LSAM && c->algorithm != LSAM_ALG_DATA_PARALLEL)
    return fail(LSAM_EINVAL, "algorithm must be LSAM_ALG_LSAM or LSAM_ALG_DATA_PARALLEL");
  if (!(c->noise_scale >= 0.f) || !std::isfinite(c->noise_scale))
    return fail(LSAM_EINVAL, "noise_scale must be finite and >= 0");
  return LSAM_OK;
}

size_t take(size_t& cursor, size_t bytes) {
  const size_t at = cursor;
  cursor = (size_t)round_up((int64_t)(cursor + bytes), 2048);   // whole 2 KiB blocks of the bf16 layout
  return at;
}

// Into how many pieces the contraction (length kd) of a layer's B x B Gram product is cut: on
// its own it has only K (B/128)^2 tiles of work for 256 compute units and a long k-loop each.
// Aims at one workgroup per compute unit (with the chip full already, two and four pieces
// measured no faster and slower), keeps at least 16 steps of 32 per piece, at most 8 pieces.
int gram_pieces(int K, int B, int kd) {
  const int64_t tiles = (int64_t)K * ((B + 127) / 128) * ((B + 127) / 128);
  const int64_t want = (256 + tiles - 1) / tiles;
  const int64_t deep = ((kd + 31) / 32) / 16;
  return (int)std::max<int64_t>(1, std::min<int64_t>({want, deep, 8}));
}

void build_layout(const lsam_config& c, Layout& lo) {
  lo.K = c.K;
  lo.L = c.n_layers;
  lo.raw = c.n_layers == 0;
  lo.B = lo.raw ? 0 : c.batch;
  lo.bf16 = !lo.raw && c.gemm_dtype == LSAM_GEMM_BF16 && c.n_conv == 0;
  lo.bf16_math = !lo.raw && c.gemm_dtype == LSAM_GEMM_BF16 && c.n_conv > 0;
  int64_t off = 0, flat = 0;
  if (lo.raw) {
    lo.d = c.d_raw;
    lo.d_pad = round_up(c.d_raw, 64);
  } else {
    lo.n_conv = c.n_conv;
    lo.preact = c.n_conv > 0 && c.preact != 0;
    // width[l]: columns of the matrix layer l reads (l < L), of the logits (l = L)
    std::vector<int> width(lo.L + 1);
    {
      int h = c.img_h, w = c.img_w;
      for (int l = 0; l <= lo.L; ++l) {
        width[l] = c.dims[l];
        if (l < lo.n_conv) {
          ConvLayer cv{};
          cv.stride = ((c.stride_mask >> l) & 1u) ? 2 : 1;
          h /= cv.stride; w /= cv.stride;
          cv.H = h; cv.W = w; cv.Cin = c.dims[l]; cv.Cout = c.dims[l + 1];
          cv.pool = (int)((c.pool_mask >> l) & 1u);
          cv.skip = ((c.skip_mask >> l) & 1u) != 0;
          if (cv.skip) {
            // the block input is what convolution l-1 read: [stride_{l-1} H_{l-1}] rows of C_{l-1} channels
            const ConvLayer& first = lo.conv[l - 1];
            cv.skip_C = first.Cin;
            cv.skip_step = first.stride * first.H / h;
            cv.proj = ((c.proj_mask >> l) & 1u) != 0;
          }
          cv.rows = (int64_t)c.batch * h * w;
          cv.ldc = (int)round_up(9 * (int64_t)cv.Cin, 8);
          lo.conv.push_back(cv);
          width[l] = 9 * cv.Cin;
          if (cv.pool) { h /= 2; w /= 2; }
        } else if (lo.n_conv > 0 && l == lo.n_conv) {
          width[l] = c.global_avg_pool ? c.dims[l] : h * w * c.dims[l];
          lo.gap_hw = c.global_avg_pool ? h * w : 0;
        }
      }
    }
    lo.ld.resize(lo.L + 1);
    for (int l = 0; l <= lo.L; ++l) lo.ld[l] = (int)round_up(width[l], 8);
    lo.need_a0 = lo.n_conv == 0 && (c.dims[0] % 8) != 0;
    for (int l = 0; l < lo.L; ++l) {
      Layer s;
      s.in = width[l];
      s.out = c.dims[l + 1];
      s.ldw = lo.ld[l];
      s.w_off = off;
      off = round_up(off + (int64_t)s.out * s.ldw, 64);
      s.b_off = off;
      off = round_up(off + s.out, 64);
      s.w_flat = flat;
      flat += (int64_t)s.out * s.in;
      s.b_flat = flat;
      flat += s.out;
      if (l < lo.n_conv && ((c.bn_mask >> l) & 1u)) {
        s.bn = true;
        s.gam_off = off;
        off = round_up(off + s.out, 64);
        s.bet_off = off;
        off = round_up(off + s.out, 64);
        s.gam_flat = flat;
        s.bet_flat = flat + s.out;
        flat += 2 * (int64_t)s.out;
      }
      lo.pieces.push_back(Piece{s.w_off, s.w_flat, s.out, s.in, s.ldw, 8 * l});
      lo.pieces.push_back(Piece{s.b_off, s.b_flat, 1, s.out, (int)round_up(s.out, 4), 8 * l + 1});
      if (s.bn) {
        lo.pieces.push_back(Piece{s.gam_off, s.gam_flat, 1, s.out, (int)round_up(s.out, 4), 8 * l + 2});
        lo.pieces.push_back(Piece{s.bet_off, s.bet_flat, 1, s.out, (int)round_up(s.out, 4), 8 * l + 3});
      }
      if (l < lo.n_conv && lo.conv[l].proj) {
        s.proj = true;
        s.proj_in = lo.conv[l].skip_C;
        s.pw_off = off;
        off = round_up(off + (int64_t)s.out * s.proj_in, 64);
        int64_t* slot[3] = {&s.pb_off, &s.pgam_off, &s.pbet_off};
        lo.pieces.push_back(Piece{s.pw_off, flat, s.out, s.proj_in, s.proj_in, 8 * l + 4});
        flat += (int64_t)s.out * s.proj_in;
        for (int q = 0; q < (lo.preact ? 1 : 3); ++q) {
          *slot[q] = off;
          lo.pieces.push_back(Piece{off, flat, 1, s.out, (int)round_up(s.out, 4), 8 * l + 5 + q});
          off = round_up(off + s.out, 64);
          flat += s.out;
        }
      }
      lo.layers.push_back(s);
    }
    lo.d = flat;
    lo.d_pad = off;
    if (lo.bf16) {
      lo.need_a0 = true;     // the input is always re-stored in the blocked layout
      lo.map.n = lo.L;
      int64_t so = 0;
      for (int l = 0; l < lo.L; ++l) {
        const Layer& ly = lo.layers[l];
        lo.shadow_off.push_back(so);
        lo.map.ldw[l] = ly.ldw;
        lo.map.cblocks[l] = b32s_blocks(ly.in);
        lo.map.begin[l] = ly.w_off;
        lo.map.end[l] = ly.w_off + (int64_t)ly.out * ly.ldw;
        lo.map.shadow[l] = so;
        so += b32s_size(ly.out, ly.in);
      }
      lo.shadow_stride = so;
    }
  }
  if (lo.raw) {
    int64_t nb = (lo.d_pad + 65535) / 65536;
    lo.nblk = (int)(nb < 1 ? 1 : (nb > 1024 ? 1024 : nb));
  } else {
    // the first backward pass leaves one partial sum of squares per workgroup that wrote a
    // piece of the gradient: room for the most any tile choice can produce
    int64_t cap = 0;
    for (const Layer& ly : lo.layers)
      cap += std::max(gemm_sumsq_capacity(ly.out, ly.in),
                      std::max(head_sumsq_slots(ly.in), ly.out / 2)) +   // ly.out / 2: first-layer kernels
             (ly.out + 63) / 64 + (ly.bn ? 2 * ((ly.out + 63) / 64) : 0) +
             (ly.proj ? gemm_sumsq_capacity(ly.out, ly.proj_in) + 2 * ((ly.out + 63) / 64) : 0);
    lo.nblk = (int)cap;
  }

  size_t cur = 0;
  const size_t vec = (size_t)lo.K * lo.d_pad * 4;
  lo.x = take(cur, vec);
  lo.v = take(cur, vec);
  lo.S = take(cur, vec);
  lo.g = lo.raw ? 0 : take(cur, vec);
  lo.xt = take(cur, lo.bf16 ? (size_t)lo.K * lo.shadow_stride * 2 : vec);
  lo.y = take(cur, (size_t)lo.d_pad * 4);
  lo.gprev = take(cur, (size_t)lo.d_pad * 4);
  if (lo.raw && c.algorithm == LSAM_ALG_DATA_PARALLEL) lo.gmean = take(cur, (size_t)lo.d_pad * 4);
  lo.partials = take(cur, (size_t)lo.K * lo.nblk * 8);
  lo.restart = take(cur, (size_t)lo.K * 4);
  lo.norms = take(cur, (size_t)lo.K * 4);
  lo.scale = take(cur, (size_t)lo.K * 4);
  lo.loss = take(cur, (size_t)lo.K * 4);
  if (!lo.raw) {
    const size_t rows = (size_t)lo.K * lo.B;
    lo.loss_rows = take(cur, rows * 4);
    lo.act.assign(lo.L + 1, 0);
    lo.dz.assign(lo.L + 1, 0);
    auto wd = [&](int l) { return l < lo.L ? lo.layers[l].in : lo.layers[lo.L - 1].out; };
    auto act_bytes = [&](int l) { return (size_t)lo.K * lo.act_elems(wd(l), lo.ld[l]) * lo.es(); };
    size_t dcol_bytes = 0;
    for (int l = 0; l < lo.n_conv; ++l) {
      ConvLayer& cv = lo.conv[l];
      const size_t full = (size_t)lo.K * cv.rows * cv.Cout * 4;
      const bool small = cv.rows < (1 << 24);      // pixel indices exact in fp32
      // the kernels that unfold on the fly, and the first layer's own, know stride 1 only
      cv.direct_in = small && cv.Cin % 32 == 0 && cv.stride == 1;
      cv.direct_dx = small && l > 0 && cv.Cout % 32 == 0 && cv.stride == 1;
      cv.first = l == 0 && cv.stride == 1 && first_conv_fits(cv.Cin, cv.Cout, cv.rows);
      if (cv.first)
        cv.first_partial = take(cur, (size_t)lo.K * first_conv_chunks(cv.rows) * cv.Cout * 32 * 4);
      else if (!cv.direct_in) cv.col = take(cur, (size_t)lo.K * cv.rows * cv.ldc * 4);
      if (cv.direct_dx) cv.wt = take(cur, (size_t)lo.K * cv.Cin * 9 * cv.Cout * 4);
      cv.out = take(cur, full);
      cv.dout = take(cur, full);
      cv.bn = lo.layers[l].bn;
      if (cv.bn) {
        cv.z = take(cur, full);
        cv.stats = take(cur, (size_t)lo.K * 2 * cv.Cout * 4);
      }
      if (cv.pool) {
        cv.pooled = take(cur, full / 4);
        cv.dpooled = take(cur, full / 4);
      }
      if (cv.proj) {
        cv.psub = take(cur, (size_t)lo.K * cv.rows * cv.skip_C * 4);
        cv.pz = take(cur, full);
        if (!lo.preact) cv.pstats = take(cur, (size_t)lo.K * 2 * cv.Cout * 4);
      }
      if (l > 0 && !cv.direct_dx) dcol_bytes = std::max(dcol_bytes, (size_t)lo.K * cv.rows * cv.ldc * 4);
    }
    if (dcol_bytes) lo.dcol = take(cur, dcol_bytes);
    if (lo.n_conv > 0) {
      size_t most = 0;
      for (const ConvLayer& cv : lo.conv)
        most = std::max(most, (size_t)lo.K * colsum_chunks(cv.rows, cv.Cout, lo.K) * cv.Cout * 4);
      for (const ConvLayer& cv : lo.conv)
        if (cv.bn) most = std::max(most, (size_t)lo.K * bn_chunks(cv.rows, cv.Cout, lo.K) * 2 * cv.Cout * 4);
      lo.colsum = take(cur, most);
    }
    // the dense layers start at n_conv; their input and its gradient are the last
    // convolution's (pooled) output and that buffer's gradient
    if (lo.n_conv > 0) {
      const ConvLayer& cv = lo.conv[lo.n_conv - 1];
      lo.act[lo.n_conv] = cv.pool ? cv.pooled : cv.out;
      lo.dz[lo.n_conv] = cv.pool ? cv.dpooled : cv.dout;
      if (lo.gap_hw) {
        lo.gap_out = take(cur, rows * lo.ld[lo.n_conv] * 4);
        lo.gap_grad = take(cur, rows * lo.ld[lo.n_conv] * 4);
        lo.act[lo.n_conv] = lo.gap_out;
        lo.dz[lo.n_conv] = lo.gap_grad;
      }
    }
    for (int l = lo.n_conv + 1; l < lo.L; ++l) lo.act[l] = take(cur, act_bytes(l));
    for (int l = lo.n_conv + 1; l <= lo.L; ++l) lo.dz[l] = take(cur, act_bytes(l));
    lo.logits = take(cur, rows * lo.ld[lo.L] * 4);
    if (lo.need_a0) lo.a0 = take(cur, act_bytes(0));
    // scratch for split-K partial sums: the largest request among this model's GEMMs
    size_t need = 0;
    for (int l = 0; l < lo.L; ++l) {
      const Layer& ly = lo.layers[l];
      if (lo.bf16) break;      // split-K serves the fp32 kernel only
      GemmDesc d{};
      d.batch = lo.K; d.in_bf16 = lo.bf16; d.bf16_math = lo.bf16_math;
      const ConvLayer* cv = l < lo.n_conv ? &lo.conv[l] : nullptr;
      const int rows = cv ? (int)cv->rows : lo.B;
      d.M = rows; d.N = ly.out; d.Kd = ly.in; d.a_kmajor = 1; d.b_kmajor = 1;     // forward
      d.out_bf16 = lo.bf16 && l + 1 < lo.L;
      d.unfold = cv && cv->direct_in ? 1 : 0;
      need = std::max(need, gemm_splitk_bytes(d));
      d.M = rows; d.N = ly.in; d.Kd = ly.out; d.a_kmajor = 1; d.b_kmajor = 0;     // dX
      d.out_bf16 = lo.bf16;
      d.unfold = 0;
      if (cv && cv->direct_dx) { d.N = cv->Cin; d.Kd = 9 * cv->Cout; d.b_kmajor = 1; d.unfold = 1; }
      if (l > 0) need = std::max(need, gemm_splitk_bytes(d));
      d.M = ly.out; d.N = ly.in; d.Kd = rows; d.a_kmajor = 0; d.b_kmajor = 0;     // dW
      d.out_bf16 = 0;
      d.unfold = cv && cv->direct_in ? 2 : 0;
      need = std::max(need, gemm_splitk_bytes(d));
      if (ly.proj) {       // the projection's three products
        d.unfold = 0;
        d.M = rows; d.N = ly.out; d.Kd = ly.proj_in; d.a_kmajor = 1; d.b_kmajor = 1;
        need = std::max(need, gemm_splitk_bytes(d));
        d.M = rows; d.N = ly.proj_in; d.Kd = ly.out; d.a_kmajor = 1; d.b_kmajor = 0;
        need = std::max(need, gemm_splitk_bytes(d));
        d.M = ly.out; d.N = ly.proj_in; d.Kd = rows; d.a_kmajor = 0; d.b_kmajor = 0;
        need = std::max(need, gemm_splitk_bytes(d));
      }
    }
    lo.splitk_bytes = need;
    if (need) lo.splitk = take(cur, need);
    if (lo.bf16) {
      // room for the most pieces any layer's Gram products are cut into
      lo.ldg = (int)round_up(lo.B, 8);
      int pieces = 1;
      for (int l = lo.n_conv; l < lo.L; ++l)
        pieces = std::max({pieces, gram_pieces(lo.K, lo.B, lo.layers[l].out), gram_pieces(lo.K, lo.B, lo.layers[l].in)});
      lo.gram1 = take(cur, (size_t)pieces * lo.K * lo.B * lo.ldg * 4);
      lo.gram2 = take(cur, (size_t)pieces * lo.K * lo.B * lo.ldg * 4);
    }
    if (c.noise_scale > 0.f) lo.noise_segs = take(cur, lo.pieces.size() * sizeof(NoiseSeg));
  }
  lo.total = cur;
}

// ---- per-kernel timing ---------------------------------------------------------------------------
enum KernelClass {
  KC_GEMM_FWD = 0, KC_GEMM_DX, KC_GEMM_DW, KC_SOFTMAX_CE, KC_BIAS_GRAD, KC_SUMSQ, KC_NORM_FINISH,
  KC_PERTURB, KC_DESCENT, KC_CENTER, KC_MISC, KC_HEAD, KC_UNFOLD, KC_POOL, KC_CONV_FIRST, KC_BATCHNORM,
  KC_GEMM_DW_STEP, KC_GEMM_DW_NORM, KC_GEMM_DW_ASCEND, KC_COUNT
};
const char* const kClassNames[KC_COUNT] = {
    "gemm_fwd", "gemm_dx", "gemm_dw", "softmax_ce", "bias_grad", "sumsq_partials", "norm_finish",
    "perturb", "descent", "center", "misc", "head", "unfold_fold", "pool", "conv_first", "batchnorm",
    "gemm_dw_step", "gemm_dw_norm", "gemm_dw_ascend"};

struct TimedLaunch {
  int cls;
  hipEvent_t a, b;
};

}  // namespace
}  // namespace lsam

namespace lsam {
void set_last_error(const char* msg) { g_err = msg ? msg : ""; }
}  // namespace lsam

using namespace lsam;

struct lsam_ctx {
  lsam_config cfg;
  std::vector<int32_t> dims, tau_explicit;
  Layout lo;
  Schedule sched;
  char* ws = nullptr;
  hipStream_t stream = nullptr;
  float lr = 0.f, rho = 0.f;
  int norm_slots = 0;   // partial sums of squares left by the last first-pass backward
  uint32_t t_step = 0;  // sampler steps taken (counter word of the Langevin noise)
  void* stage = nullptr;   // pinned host staging buffer for the read-out / restore calls (lazy)
  NoiseMap noise{};     // where the Langevin noise goes; used when cfg.noise_scale > 0
  bool fuse_step = true;   // take the sampler step inside the second pass's dW epilogues where possible
  // timing
  bool timing = false;
  std::vector<TimedLaunch> pending;
  std::vector<hipEvent_t> free_events;
  int64_t t_count[KC_COUNT] = {0};
  double t_ms[KC_COUNT] = {0};

  template <typename T> T* at(size_t off) const { return reinterpret_cast<T*>(ws + off); }
};

namespace {

struct LaunchTimer {
  lsam_ctx* c;
  TimedLaunch t;
  bool on;
  LaunchTimer(lsam_ctx* ctx, int cls) : c(ctx), on(ctx->timing) {
    if (!on) return;
    t.cls = cls;
    t.a = grab();
    t.b = grab();
    if (t.a == nullptr || t.b == nullptr) { on = false; return; }
    (void)hipEventRecord(t.a, c->stream);
  }
  ~LaunchTimer() {
    if (!on) return;
    (void)hipEventRecord(t.b, c->stream);
    c->pending.push_back(t);
  }
  hipEvent_t grab() {
    if (!c->free_events.empty()) {
      hipEvent_t e = c->free_events.back();
      c->free_events.pop_back();
      return e;
    }
    hipEvent_t e = nullptr;
    if (hipEventCreate(&e) != hipSuccess) return nullptr;
    return e;
  }
};

int drain_timing(lsam_ctx* c) {
  if (c->pending.empty()) return LSAM_OK;
  HIP_TRY(hipStreamSynchronize(c->stream));
  for (auto& t : c->pending) {
    float ms = 0.f;
    if (hipEventElapsedTime(&ms, t.a, t.b) == hipSuccess) {
      c->t_ms[t.cls] += ms;
      c->t_count[t.cls] += 1;
    }
    c->free_events.push_back(t.a);
    c->free_events.push_back(t.b);
  }
  c->pending.clear();
  return LSAM_OK;
}

int check_launch(const char* what) {
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return fail(LSAM_EHIP, "launch of %s failed: %s", what, hipGetErrorString(e));
  return LSAM_OK;
}

float coupling(const lsam_ctx* c, int i) {
  if (c->cfg.algorithm == LSAM_ALG_DATA_PARALLEL) return 0.f;
  if (c->cfg.lambda_abs >= 0.f) return c->cfg.lambda_abs;
  return (float)((double)c->cfg.lambda0 / ((double)c->lr * (double)c->sched.tau()[i]));
}

// Split-K scratch shared by all GEMMs of a step.
void split(const lsam_ctx* c, GemmDesc& d) {
  d.splitk_ws = c->lo.splitk_bytes ? c->at<float>(c->lo.splitk) : nullptr;
  d.splitk_bytes = c->lo.splitk_bytes;
  d.bf16_math = c->lo.bf16_math;     // every GEMM of a step shares the arithmetic mode, too
}

// Forward pass of the convolution layers: unfold, GEMM with bias + ReLU, pool.  `params`: x or
// the perturbed copy (fp32).  The result is the dense layers' input, lo.act[n_conv].
int conv_forward(lsam_ctx* c, const float* X, const float* params) {
  const Layout& lo = c->lo;
  hipStream_t s = c->stream;
  const float* in = X;
  for (int l = 0; l < lo.n_conv; ++l) {
    const ConvLayer& cv = lo.conv[l];
    const Layer& ly = lo.layers[l];
    float* col = cv.direct_in ? nullptr : c->at<float>(cv.col);
    if (cv.first) {
      LaunchTimer t(c, KC_CONV_FIRST);
      if (launch_first_conv_forward(in, params, lo.d_pad, ly.w_off, ly.b_off, ly.ldw,
                                    c->at<float>(cv.bn ? cv.z : cv.out), cv.bn ? 0 : 1,
                                    lo.bf16_math ? 1 : 0, lo.K, cv.rows, cv.H, cv.W, cv.Cin, cv.Cout,
                                    s) != 0)
        return fail(LSAM_EINVAL, "first convolution rejected");
    } else if (!cv.direct_in) {
      LaunchTimer t(c, KC_UNFOLD);
      if (launch_unfold3x3(in, cv.rows * cv.stride * cv.stride * cv.Cin, col, cv.rows * cv.ldc, cv.ldc,
                           lo.K, lo.B, cv.H, cv.W, cv.Cin, cv.stride, s) != 0)
        return fail(LSAM_EINVAL, "unfold of convolution %d rejected", l);
    }
    if (!cv.first) {
      GemmDesc d{};
      d.A = col; d.strideA = cv.rows * cv.ldc; d.ldA = cv.ldc; d.a_kmajor = 1;
      if (cv.direct_in) {
        d.A = in; d.strideA = cv.rows * cv.Cin; d.ldA = cv.Cin;
        d.unfold = 1; d.unfold_C = cv.Cin; d.unfold_H = cv.H; d.unfold_W = cv.W;
      }
      d.B = params + ly.w_off; d.strideB = lo.d_pad; d.ldB = ly.ldw; d.b_kmajor = 1;
      d.C = c->at<float>(cv.bn ? cv.z : cv.out); d.strideC = cv.rows * cv.Cout; d.ldC = cv.Cout;
      d.M = (int)cv.rows; d.N = cv.Cout; d.Kd = ly.in; d.batch = lo.K;
      d.epilogue = cv.bn ? EPI_BIAS : EPI_BIAS_RELU;
      d.bias = params + ly.b_off; d.strideBias = lo.d_pad;
      split(c, d);
      LaunchTimer t(c, KC_GEMM_FWD);
      if (launch_gemm(d, s) != 0) return fail(LSAM_EINVAL, "forward GEMM of convolution %d rejected", l);
    }
    if (cv.proj) {
      // projection shortcut: the block input's pixels (every second one if the block halved
      // the image) through a 1x1 convolution, then that output's own statistics
      const ConvLayer& src = lo.conv[l - 2];
      const float* sub = c->at<float>(src.out);
      if (cv.skip_step == 2) {
        LaunchTimer t(c, KC_UNFOLD);
        if (launch_subsample2(sub, c->at<float>(cv.psub), (int64_t)lo.K * lo.B, cv.H, cv.W, cv.skip_C, s) != 0)
          return fail(LSAM_EINVAL, "projection of convolution %d: gather rejected", l);
        sub = c->at<float>(cv.psub);
      }
      GemmDesc d{};
      d.A = sub; d.strideA = cv.rows * cv.skip_C; d.ldA = cv.skip_C; d.a_kmajor = 1;
      d.B = params + ly.pw_off; d.strideB = lo.d_pad; d.ldB = ly.proj_in; d.b_kmajor = 1;
      d.C = c->at<float>(cv.pz); d.strideC = cv.rows * cv.Cout; d.ldC = cv.Cout;
      d.M = (int)cv.rows; d.N = cv.Cout; d.Kd = ly.proj_in; d.batch = lo.K;
      d.epilogue = EPI_BIAS;
      d.bias = params + ly.pb_off; d.strideBias = lo.d_pad;
      split(c, d);
      {
        LaunchTimer t(c, KC_GEMM_FWD);
        if (launch_gemm(d, s) != 0) return fail(LSAM_EINVAL, "projection of convolution %d rejected", l);
      }
      if (lo.preact) {
        // the bare projection joins the convolution's output in front of the normalisation
        LaunchTimer t(c, KC_POOL);
        if (launch_add_into(c->at<float>(cv.z), c->at<float>(cv.pz), (int64_t)lo.K * cv.rows * cv.Cout, s) != 0)
          return fail(LSAM_EINVAL, "projection of convolution %d: sum rejected", l);
      } else {
        LaunchTimer t(c, KC_BATCHNORM);
        if (launch_bn_stats(c->at<float>(cv.pz), c->at<float>(lo.colsum), c->at<float>(cv.pstats), lo.K,
                            cv.rows, cv.Cout, c->cfg.bn_eps, s) != 0)
          return fail(LSAM_EINVAL, "projection of convolution %d: statistics rejected", l);
      }
    } else if (cv.skip && lo.preact) {
      // identity shortcut of a pre-activation block: the sum two convolutions below
      LaunchTimer t(c, KC_POOL);
      if (launch_add_into(c->at<float>(cv.z), c->at<float>(lo.conv[l - 2].z), (int64_t)lo.K * cv.rows * cv.Cout,
                          s) != 0)
        return fail(LSAM_EINVAL, "shortcut of convolution %d: sum rejected", l);
    }
    if (cv.bn) {
      LaunchTimer t(c, KC_BATCHNORM);
      ShortcutDesc sc{};
      const bool post_sum = cv.skip && !lo.preact;     // the shortcut joins behind the normalisation
      if (post_sum && cv.proj) {
        sc.pz = c->at<float>(cv.pz); sc.pstats = c->at<float>(cv.pstats);
        sc.pgam_off = ly.pgam_off; sc.pbet_off = ly.pbet_off;
      } else if (post_sum) {
        // the block input: what convolution l-1 read, i.e. the ReLU output of convolution l-2
        sc.src = c->at<float>(lo.conv[l - 2].out);
        sc.stride = lo.conv[l - 2].rows * cv.skip_C;
        sc.H = cv.H; sc.W = cv.W; sc.Cs = cv.skip_C; sc.step = cv.skip_step;
      }
      if (launch_bn_forward(c->at<float>(cv.z), c->at<float>(lo.colsum), c->at<float>(cv.stats), params,
                            lo.d_pad, ly.gam_off, ly.bet_off, c->at<float>(cv.out), lo.K, cv.rows,
                            cv.Cout, c->cfg.bn_eps, post_sum ? &sc : nullptr, s) != 0)
        return fail(LSAM_EINVAL, "batch normalisation of convolution %d rejected", l);
    }
    in = c->at<float>(cv.out);
    if (cv.pool) {
      LaunchTimer t(c, KC_POOL);
      if (launch_maxpool2(in, c->at<float>(cv.pooled), (int64_t)lo.K * lo.B, cv.H, cv.W, cv.Cout, s) != 0)
        return fail(LSAM_EINVAL, "pool of convolution %d rejected", l);
      in = c->at<float>(cv.pooled);
    }
  }
  if (lo.gap_hw) {
    LaunchTimer t(c, KC_POOL);
    const ConvLayer& cv = lo.conv[lo.n_conv - 1];
    if (launch_avgpool(in, c->at<float>(lo.gap_out), (int64_t)lo.K * lo.B, lo.gap_hw, cv.Cout,
                       lo.ld[lo.n_conv], s) != 0)
      return fail(LSAM_EINVAL, "global average pooling rejected");
  }
  return LSAM_OK;
}

// Backward pass of the convolution layers.  On entry lo.dz[n_conv] holds the gradient of the
// dense layers' input (already zero where that input is zero).  Appends the layers' partial
// sums of squares at ssq[*slots...] when ssq is non-null.
int conv_backward(lsam_ctx* c, const float* X, const float* params, double* ssq, int* slots) {
  const Layout& lo = c->lo;
  hipStream_t s = c->stream;
  float* g = c->at<float>(lo.g);
  if (lo.gap_hw) {
    // the pooled vector's gradient goes back to every position, through the ReLU the image came
    // from unless a pool sits in between (whose backward pass applies that mask)
    LaunchTimer t(c, KC_POOL);
    const ConvLayer& cv = lo.conv[lo.n_conv - 1];
    if (launch_avgpool_backward(c->at<float>(lo.gap_grad), cv.pool ? nullptr : c->at<float>(cv.out),
                                c->at<float>(cv.pool ? cv.dpooled : cv.dout), (int64_t)lo.K * lo.B,
                                lo.gap_hw, cv.Cout, lo.ld[lo.n_conv], s) != 0)
      return fail(LSAM_EINVAL, "global average pooling (backward) rejected");
  }
  for (int l = lo.n_conv - 1; l >= 0; --l) {
    const ConvLayer& cv = lo.conv[l];
    const Layer& ly = lo.layers[l];
    float* dout = c->at<float>(cv.dout);
    // room for every partial sum of squares this layer's kernels may write, checked up front
    if (ssq && *slots + std::max(gemm_sumsq_capacity(ly.out, ly.in), ly.out / 2) + (ly.out + 63) / 64 +
                       (ly.bn ? 2 * ((ly.out + 63) / 64) : 0) +
                       (ly.proj ? gemm_sumsq_capacity(ly.out, ly.proj_in) + 2 * ((ly.out + 63) / 64) : 0) > lo.nblk)
      return fail(LSAM_ESTATE, "gradient-norm partials would overrun their buffer at convolution %d", l);
    if (cv.pool) {
      LaunchTimer t(c, KC_POOL);
      if (launch_maxpool2_backward(c->at<float>(cv.out), c->at<float>(cv.dpooled), dout,
                                   (int64_t)lo.K * lo.B, cv.H, cv.W, cv.Cout, s) != 0)
        return fail(LSAM_EINVAL, "pool backward of convolution %d rejected", l);
    }
    if (cv.bn) {
      // dout holds the gradient behind the ReLU; turn it into the gradient of the convolution's
      // output and leave dgamma, dbeta in g
      LaunchTimer t(c, KC_BATCHNORM);
      float* part = c->at<float>(lo.colsum);
      const int chunks = launch_bn_backward_partials(c->at<float>(cv.z), dout, c->at<float>(cv.stats),
                                                     part, lo.K, cv.rows, cv.Cout, s);
      if (chunks < 0) return fail(LSAM_EINVAL, "batch normalisation of convolution %d rejected", l);
      if (ly.bet_off == ly.gam_off + cv.Cout) {
        // gamma and beta are neighbours in the layout (64 | C_out): one sum over both halves
        const int used = launch_bias_grad(part, 2 * cv.Cout, 0, g + ly.gam_off, lo.d_pad, lo.K, chunks,
                                          2 * cv.Cout, ssq ? ssq + *slots : nullptr, lo.nblk, s);
        if (ssq) *slots += used;
      } else {
        int used = launch_bias_grad(part, 2 * cv.Cout, 0, g + ly.gam_off, lo.d_pad, lo.K, chunks,
                                    cv.Cout, ssq ? ssq + *slots : nullptr, lo.nblk, s);
        if (ssq) *slots += used;
        used = launch_bias_grad(part + cv.Cout, 2 * cv.Cout, 0, g + ly.bet_off, lo.d_pad, lo.K, chunks,
                                cv.Cout, ssq ? ssq + *slots : nullptr, lo.nblk, s);
        if (ssq) *slots += used;
      }
      // A block's closing convolution keeps dY: it is also the gradient of the shortcut, added
      // to the block input's gradient further down.  Its dZ goes where Z was (Z is not needed again).
      float* dz = (cv.skip && !lo.preact) ? c->at<float>(cv.z) : dout;
      launch_bn_backward_apply(c->at<float>(cv.z), dout, dz, c->at<float>(cv.stats), params, g, lo.d_pad,
                               ly.gam_off, ly.bet_off, lo.K, cv.rows, cv.Cout, s);
      if (cv.proj && !lo.preact) {
        // the same gradient dY enters the projection's normalisation: dgamma_p, dbeta_p, then
        // the gradient of the 1x1 convolution's output, which takes that output's place
        float* pz = c->at<float>(cv.pz);
        const int pchunks = launch_bn_backward_partials(pz, dout, c->at<float>(cv.pstats), part, lo.K,
                                                        cv.rows, cv.Cout, s);
        if (pchunks < 0) return fail(LSAM_EINVAL, "projection of convolution %d: normalisation rejected", l);
        int used = launch_bias_grad(part, 2 * cv.Cout, 0, g + ly.pgam_off, lo.d_pad, lo.K, pchunks, cv.Cout,
                                    ssq ? ssq + *slots : nullptr, lo.nblk, s);
        if (ssq) *slots += used;
        used = launch_bias_grad(part + cv.Cout, 2 * cv.Cout, 0, g + ly.pbet_off, lo.d_pad, lo.K, pchunks,
                                cv.Cout, ssq ? ssq + *slots : nullptr, lo.nblk, s);
        if (ssq) *slots += used;
        launch_bn_backward_apply(pz, dout, pz, c->at<float>(cv.pstats), params, g, lo.d_pad, ly.pgam_off,
                                 ly.pbet_off, lo.K, cv.rows, cv.Cout, s);
      }
      dout = dz;
    }
    if (lo.preact && l + 2 < lo.n_conv && lo.conv[l + 2].skip && !lo.conv[l + 2].proj) {
      // this convolution's sum is the identity shortcut of the block above: that block's sum
      // hands its gradient (complete since its own backward pass) down unchanged
      LaunchTimer t(c, KC_POOL);
      if (launch_add_into(dout, c->at<float>(lo.conv[l + 2].dout), (int64_t)lo.K * cv.rows * cv.Cout, s) != 0)
        return fail(LSAM_EINVAL, "shortcut into convolution %d: sum rejected", l);
    }
    if (cv.proj) {
      // dW_p = dZ_p^T S and dS = dZ_p W_p; dS replaces the gathered pixels and reaches the block
      // input's gradient once the block's opening convolution has written that gradient.  In a
      // pre-activation block the projection's output gradient is the sum's own.
      const float* dzp = lo.preact ? dout : c->at<float>(cv.pz);
      float* psub = c->at<float>(cv.psub);
      {
        GemmDesc d{};
        d.A = dzp; d.strideA = cv.rows * cv.Cout; d.ldA = cv.Cout; d.a_kmajor = 0;
        d.B = cv.skip_step == 2 ? psub : c->at<float>(lo.conv[l - 2].out);
        d.strideB = cv.rows * cv.skip_C; d.ldB = cv.skip_C; d.b_kmajor = 0;
        d.C = g + ly.pw_off; d.strideC = lo.d_pad; d.ldC = ly.proj_in;
        d.M = cv.Cout; d.N = ly.proj_in; d.Kd = (int)cv.rows; d.batch = lo.K;
        d.epilogue = EPI_PLAIN;
        split(c, d);
        if (ssq) { d.sumsq = ssq + *slots; d.sumsq_stride = lo.nblk; }
        int used = 0;
        LaunchTimer t(c, KC_GEMM_DW);
        if (launch_gemm(d, s, &used) != 0) return fail(LSAM_EINVAL, "projection of convolution %d: dW rejected", l);
        if (ssq) *slots += used;
      }
      GemmDesc d{};
      d.A = dzp; d.strideA = cv.rows * cv.Cout; d.ldA = cv.Cout; d.a_kmajor = 1;
      d.B = params + ly.pw_off; d.strideB = lo.d_pad; d.ldB = ly.proj_in; d.b_kmajor = 0;
      d.C = psub; d.strideC = cv.rows * cv.skip_C; d.ldC = cv.skip_C;
      d.M = (int)cv.rows; d.N = ly.proj_in; d.Kd = cv.Cout; d.batch = lo.K;
      d.epilogue = EPI_PLAIN;
      split(c, d);
      LaunchTimer t(c, KC_GEMM_DX);
      if (launch_gemm(d, s) != 0) return fail(LSAM_EINVAL, "projection of convolution %d: dX rejected", l);
    }
    if (cv.first) {
      LaunchTimer t(c, KC_CONV_FIRST);
      const int used = launch_first_conv_wgrad(X, dout, c->at<float>(cv.first_partial), g, lo.d_pad,
                                               ly.w_off, ly.b_off, ly.ldw, lo.bf16_math ? 1 : 0,
                                               (lo.bf16_math || cv.bn) ? 1 : 0, lo.K,
                                               cv.rows, cv.H, cv.W, cv.Cin, cv.Cout,
                                               ssq ? ssq + *slots : nullptr, lo.nblk, s);
      if (used < 0) return fail(LSAM_EINVAL, "first convolution's weight gradient rejected");
      if (ssq) *slots += used;
      if (!lo.bf16_math) continue;    // otherwise the bias gradient is still to come, below
    }
    if (!cv.first)
    {
      GemmDesc d{};
      d.A = dout; d.strideA = cv.rows * cv.Cout; d.ldA = cv.Cout; d.a_kmajor = 0;
      d.B = c->at<float>(cv.col); d.strideB = cv.rows * cv.ldc; d.ldB = cv.ldc; d.b_kmajor = 0;
      if (cv.direct_in) {
        d.B = l == 0 ? X : c->at<float>(lo.conv[l - 1].pool ? lo.conv[l - 1].pooled : lo.conv[l - 1].out);
        d.strideB = cv.rows * cv.Cin; d.ldB = cv.Cin;
        d.unfold = 2; d.unfold_C = cv.Cin; d.unfold_H = cv.H; d.unfold_W = cv.W;
      }
      d.C = g + ly.w_off; d.strideC = lo.d_pad; d.ldC = ly.ldw;
      d.M = cv.Cout; d.N = ly.in; d.Kd = (int)cv.rows; d.batch = lo.K;
      d.epilogue = EPI_PLAIN;
      split(c, d);
      if (ssq) { d.sumsq = ssq + *slots; d.sumsq_stride = lo.nblk; }
      int used = 0;
      LaunchTimer t(c, KC_GEMM_DW);
      if (launch_gemm(d, s, &used) != 0) return fail(LSAM_EINVAL, "dW GEMM of convolution %d rejected", l);
      if (ssq) *slots += used;
    }
    // The bias of a normalised convolution has no influence on the loss: its gradient, the
    // column sums of dZ = gamma/sigma (dY - mean dY - Xh mean(dY Xh)), is zero because Xh sums
    // to zero.  It is left at the zero the gradient buffer starts from instead of being summed
    // up as rounding noise.
    if (!cv.bn) {
      // bias gradient: column sums of dout, in two fixed-order stages
      LaunchTimer t(c, KC_BIAS_GRAD);
      const int chunks = launch_colsum_partials(dout, cv.rows, cv.Cout, lo.K, c->at<float>(lo.colsum), s);
      if (chunks < 0) return fail(LSAM_EINVAL, "bias gradient of convolution %d rejected", l);
      const int used = launch_bias_grad(c->at<float>(lo.colsum), cv.Cout, 0, g + ly.b_off, lo.d_pad,
                                        lo.K, chunks, cv.Cout, ssq ? ssq + *slots : nullptr, lo.nblk, s);
      if (ssq) *slots += used;
    }
    if (l > 0 && cv.direct_dx) {
      // dX as a convolution of the output gradient with the mirrored filters, written straight
      // into the gradient of the image this layer read (masked by the ReLU output it came
      // from when no pool sits in between; a pool's backward pass applies the mask itself)
      const ConvLayer& below = lo.conv[l - 1];
      float* wt = c->at<float>(cv.wt);
      {
        LaunchTimer t(c, KC_MISC);
        launch_flip_filters(params + ly.w_off, lo.d_pad, ly.ldw, wt, lo.K, cv.Cout, cv.Cin, s);
      }
      GemmDesc d{};
      d.A = dout; d.strideA = cv.rows * cv.Cout; d.ldA = cv.Cout; d.a_kmajor = 1;
      d.unfold = 1; d.unfold_C = cv.Cout; d.unfold_H = cv.H; d.unfold_W = cv.W;
      d.B = wt; d.strideB = (int64_t)cv.Cin * 9 * cv.Cout; d.ldB = 9 * cv.Cout; d.b_kmajor = 1;
      d.C = c->at<float>(below.pool ? below.dpooled : below.dout);
      d.strideC = cv.rows * cv.Cin; d.ldC = cv.Cin;
      d.M = (int)cv.rows; d.N = cv.Cin; d.Kd = 9 * cv.Cout; d.batch = lo.K;
      d.epilogue = below.pool ? EPI_PLAIN : EPI_MASK;
      if (!below.pool) {
        d.mask = c->at<float>(below.out); d.strideMask = cv.rows * cv.Cin; d.ldMask = cv.Cin;
      }
      split(c, d);
      LaunchTimer t(c, KC_GEMM_DX);
      if (launch_gemm(d, s) != 0) return fail(LSAM_EINVAL, "dX GEMM of convolution %d rejected", l);
    } else if (l > 0) {
      const ConvLayer& below = lo.conv[l - 1];
      float* dcol = c->at<float>(lo.dcol);
      {
        GemmDesc d{};
        d.A = dout; d.strideA = cv.rows * cv.Cout; d.ldA = cv.Cout; d.a_kmajor = 1;
        d.B = params + ly.w_off; d.strideB = lo.d_pad; d.ldB = ly.ldw; d.b_kmajor = 0;
        d.C = dcol; d.strideC = cv.rows * cv.ldc; d.ldC = cv.ldc;
        d.M = (int)cv.rows; d.N = ly.in; d.Kd = cv.Cout; d.batch = lo.K;
        d.epilogue = EPI_PLAIN;
        split(c, d);
        LaunchTimer t(c, KC_GEMM_DX);
        if (launch_gemm(d, s) != 0) return fail(LSAM_EINVAL, "dX GEMM of convolution %d rejected", l);
      }
      // the image this layer read is the layer below's pooled output (its gradient then still
      // has to pass that pool and ReLU) or its ReLU output (masked here)
      LaunchTimer t(c, KC_UNFOLD);
      if (launch_fold3x3(dcol, cv.rows * cv.ldc, cv.ldc,
                         c->at<float>(below.pool ? below.dpooled : below.dout),
                         below.pool ? nullptr : c->at<float>(below.out),
                         cv.rows * cv.stride * cv.stride * cv.Cin, lo.K, lo.B, cv.H, cv.W, cv.Cin,
                         cv.stride, s) != 0)
        return fail(LSAM_EINVAL, "fold of convolution %d rejected", l);
    }
    if (l + 1 < lo.n_conv && lo.conv[l + 1].skip && (lo.conv[l + 1].proj || !lo.preact)) {
      // this convolution opened a residual block: the gradient of the block output (kept by the
      // closing convolution) also reaches the block input through the shortcut
      const ConvLayer& top = lo.conv[l + 1];
      const ConvLayer& below = lo.conv[l - 1];
      const ShortcutDesc sc{nullptr, below.rows * top.skip_C, top.H, top.W, top.skip_C, top.skip_step};
      LaunchTimer t(c, KC_POOL);
      if (launch_shortcut_backward(c->at<float>(top.proj ? top.psub : top.dout), c->at<float>(below.dout),
                                   c->at<float>(below.out), sc, lo.K, top.rows,
                                   top.proj ? top.skip_C : top.Cout, s) != 0)
        return fail(LSAM_EINVAL, "shortcut of the block closed by convolution %d rejected", l + 1);
    }
  }
  return LSAM_OK;
}

// Whether the narrow-classifier-head kernels serve the last layer (fp32 dense arithmetic only).
bool head_is_fused(const Layout& lo) {
  return !lo.raw && !lo.bf16 && !lo.bf16_math &&
         head_fits(lo.B, lo.layers[lo.L - 1].out, lo.layers[lo.L - 1].in);
}

// Whether the norm of a layer's unsaved first-pass weight gradient comes from the Gram matrices
// of its factors: when they take at most half the flops of the product itself.
bool gram_norm_pays(int B, int out, int in) {
  return 2 * (int64_t)B * (out + in) <= (int64_t)out * in;
}

// forward + backward of all replicas; weights taken from `wts` (fp32 or bf16 per mode).
// `second` selects the pass at the perturbed point: its biases are x_b + scale * g1_b, which in
// fp32 mode sit in the perturbed copy and in bf16 mode are formed in the GEMM epilogue from
// the fp32 master bias and the first-pass bias gradient (only matrix operands are rounded).
// With convolution layers (fp32) the dense layers are l0 = n_conv .. L-1 and read what the
// convolution stack produced.
int forward_backward(lsam_ctx* c, const void* X, const int32_t* labels, const void* wts,
                     bool second, bool fuse_norm, const SamplerFusion* fuse = nullptr,
                     bool norm_only = false) {
  const bool want_loss = !second;
  const Layout& lo = c->lo;
  const int K = lo.K, B = lo.B, L = lo.L, l0 = lo.n_conv;
  const int bf = lo.bf16 ? 1 : 0;
  hipStream_t s = c->stream;
  const float* params = static_cast<const float*>(wts);   // fp32 mode: x or the perturbed copy
  const void* A0 = X;
  if (l0 > 0) {
    int rc = conv_forward(c, static_cast<const float*>(X), params);
    if (rc != LSAM_OK) return rc;
    A0 = c->at<char>(lo.act[l0]);
  }
  // weight matrix l as a GEMM operand: fp32 rows inside the flat vector, or its blocked bf16 copy
  auto wptr = [&](int l) {
    return bf ? (const char*)wts + (size_t)lo.shadow_off[l] * 2
              : (const char*)wts + (size_t)lo.layers[l].w_off * 4;
  };
  const int64_t wstride = bf ? lo.shadow_stride : lo.d_pad;
  auto width = [&](int l) { return l < L ? lo.layers[l].in : lo.layers[L - 1].out; };
  auto astride = [&](int l) { return lo.act_elems(width(l), lo.ld[l]); };

  // A narrow fp32 classifier head is not run as GEMMs: two fused kernels cover its forward
  // pass, the loss, dZ, dX, dW and db.
  const bool head = head_is_fused(lo);
  for (int l = l0; l < (head ? L - 1 : L); ++l) {
    const Layer& ly = lo.layers[l];
    const bool last = l == L - 1;
    GemmDesc d{};
    d.b32s = bf;
    d.A = l == l0 ? A0 : c->at<char>(lo.act[l]);
    d.strideA = astride(l); d.ldA = lo.ld[l]; d.a_kmajor = 1; d.cbA = b32s_blocks(ly.in);
    d.B = wptr(l); d.strideB = wstride; d.ldB = ly.ldw; d.b_kmajor = 1; d.cbB = b32s_blocks(ly.in);
    d.C = last ? c->at<char>(lo.logits) : c->at<char>(lo.act[l + 1]);
    d.strideC = last ? (int64_t)B * lo.ld[l + 1] : astride(l + 1); d.ldC = lo.ld[l + 1];
    d.cbC = b32s_blocks(ly.out);
    d.M = B; d.N = ly.out; d.Kd = ly.in; d.batch = K;
    d.in_bf16 = bf; d.out_bf16 = bf && !last;
    d.epilogue = last ? EPI_BIAS : EPI_BIAS_RELU;
    d.bias = c->at<float>(lo.x) + ly.b_off; d.strideBias = lo.d_pad;
    if (second && !bf) d.bias = c->at<float>(lo.xt) + ly.b_off;
    if (second && bf) {
      d.bias_dir = c->at<float>(lo.g) + ly.b_off;
      d.bias_scale = c->at<float>(lo.scale);
    }
    split(c, d);
    LaunchTimer t(c, KC_GEMM_FWD);
    if (launch_gemm(d, s) != 0) return fail(LSAM_EINVAL, "forward GEMM of layer %d rejected", l);
  }
  // the gradient of the first dense layer's input is needed when convolutions sit below it
  const bool need_dA0 = l0 > 0;
  if (head) {
    const Layer& ly = lo.layers[L - 1];
    const float* in_act = L - 1 == l0 ? static_cast<const float*>(A0) : c->at<float>(lo.act[L - 1]);
    LaunchTimer t(c, KC_HEAD);
    if (launch_head_forward_backward(in_act, params + ly.w_off, params + ly.b_off, lo.d_pad, labels,
                                     c->at<float>(lo.dz[L]), lo.ld[L],
                                     want_loss ? c->at<float>(lo.loss_rows) : nullptr,
                                     (L - 1 > l0 || need_dA0) ? c->at<float>(lo.dz[L - 1]) : nullptr,
                                     K, B, ly.out, ly.in, s) != 0)
      return fail(LSAM_EHIP, "classifier-head kernel could not be launched");
  } else {
    LaunchTimer t(c, KC_SOFTMAX_CE);
    launch_softmax_ce(c->at<float>(lo.logits), lo.ld[L], labels, c->at<char>(lo.dz[L]),
                      bf ? astride(L) : (int64_t)lo.ld[L], bf,
                      want_loss ? c->at<float>(lo.loss_rows) : nullptr, K, B, lo.layers[L - 1].out, s);
  }
  float* g = c->at<float>(lo.g);
  // first pass: the kernels that write the gradient also leave the partial sums of its squares
  double* ssq = fuse_norm ? c->at<double>(lo.partials) : nullptr;
  int slots = 0;
  for (int l = L - 1; l >= l0; --l) {
    const Layer& ly = lo.layers[l];
    const char* dz = c->at<char>(lo.dz[l + 1]);
    const int ld_dz = lo.ld[l + 1];
    const void* act = l == l0 ? A0 : (const void*)c->at<char>(lo.act[l]);
    // the layer's kernels may write this many partial sums of squares: checked before they run
    if (ssq && slots + std::max(gemm_sumsq_capacity(ly.out, ly.in), head_sumsq_slots(ly.in)) +
                       (ly.out + 63) / 64 > lo.nblk)
      return fail(LSAM_ESTATE, "gradient-norm partials would overrun their buffer at layer %d", l);
    if (head && l == L - 1) {
      LaunchTimer t(c, KC_HEAD);
      const int used = launch_head_weight_grad(
          reinterpret_cast<const float*>(dz), ld_dz, static_cast<const float*>(act), lo.ld[l],
          g + ly.w_off, ly.ldw, g + ly.b_off, lo.d_pad, K, B, ly.out, ly.in,
          ssq ? ssq + slots : nullptr, lo.nblk, s);
      if (ssq) slots += used;
      continue;
    }
    auto weight_grad = [&]() -> int {
      GemmDesc d{};
      d.b32s = bf;
      d.A = dz; d.strideA = astride(l + 1); d.ldA = ld_dz; d.a_kmajor = 0; d.cbA = b32s_blocks(ly.out);
      d.B = act; d.strideB = astride(l); d.ldB = lo.ld[l]; d.b_kmajor = 0; d.cbB = b32s_blocks(ly.in);
      d.C = g + ly.w_off; d.strideC = lo.d_pad; d.ldC = ly.ldw;
      d.M = ly.out; d.N = ly.in; d.Kd = B; d.batch = K;
      d.in_bf16 = bf; d.out_bf16 = 0; d.epilogue = EPI_PLAIN;
      split(c, d);
      if (ssq) { d.sumsq = ssq + slots; d.sumsq_stride = lo.nblk; }
      d.sumsq_only = (ssq && norm_only) ? 1 : 0;   // the gradient itself is recomputed by ascend_pass
      // Of a gradient that is not stored only the norm is wanted, and ||dZ^T A||_F^2 is the inner
      // product of the B x B Gram matrices dZ dZ^T and A A^T: 2 B^2 (out + in) flops instead of
      // 2 B out in.  Taken when that is at most half the work.
      if (d.sumsq_only && gram_norm_pays(B, ly.out, ly.in)) {
        LaunchTimer t(c, KC_GEMM_DW_NORM);
        for (int which = 0; which < 2; ++which) {
          GemmDesc q{};
          q.b32s = 1;
          q.A = q.B = which == 0 ? (const void*)dz : act;
          q.strideA = q.strideB = which == 0 ? astride(l + 1) : astride(l);
          q.ldA = q.ldB = which == 0 ? ld_dz : lo.ld[l];
          q.a_kmajor = q.b_kmajor = 1;
          q.cbA = q.cbB = b32s_blocks(which == 0 ? ly.out : ly.in);
          q.C = c->at<float>(which == 0 ? lo.gram1 : lo.gram2);
          q.strideC = (int64_t)B * lo.ldg; q.ldC = lo.ldg;
          q.M = q.N = B; q.Kd = which == 0 ? ly.out : ly.in; q.batch = K;
          q.in_bf16 = 1; q.out_bf16 = 0; q.epilogue = EPI_PLAIN;
          q.ksplit = gram_pieces(K, B, q.Kd); q.split_stride = (int64_t)K * B * lo.ldg;
          if (launch_gemm(q, s) != 0) return fail(LSAM_EINVAL, "Gram GEMM of layer %d rejected", l);
        }
        slots += launch_gram_dot(c->at<float>(lo.gram1), c->at<float>(lo.gram2), (int64_t)B * lo.ldg,
                                 (int64_t)B * lo.ldg, K, gram_pieces(K, B, ly.out), gram_pieces(K, B, ly.in),
                                 (int64_t)K * B * lo.ldg, ssq + slots, lo.nblk, s);
        return LSAM_OK;
      }
      SamplerFusion f;
      if (fuse) {
        // this layer's share of the sampler step happens in the epilogue: W_l of x, v, S, y
        f = *fuse;
        f.x += ly.w_off; f.v += ly.w_off; f.S += ly.w_off; f.y += ly.w_off;
        f.shadow += lo.shadow_off[l];
        f.cbShadow = b32s_blocks(ly.in);
        d.fuse = &f;
      }
      int used = 0;
      LaunchTimer t(c, fuse ? KC_GEMM_DW_STEP : d.sumsq_only ? KC_GEMM_DW_NORM : KC_GEMM_DW);
      if (launch_gemm(d, s, &used) != 0) return fail(LSAM_EINVAL, "dW GEMM of layer %d rejected", l);
      if (ssq) slots += used;
      return LSAM_OK;
    };
    auto bias_grad = [&]() {
      {
        LaunchTimer t(c, KC_BIAS_GRAD);
        const int used = launch_bias_grad(dz, bf ? astride(l + 1) : (int64_t)ld_dz, bf, g + ly.b_off,
                                          lo.d_pad, K, B, ly.out, ssq ? ssq + slots : nullptr,
                                          lo.nblk, s);
        if (ssq) slots += used;
      }
      if (fuse) {
        // the bias vector's share of the sampler step (the slot of b_l is padded to 64 floats
        // with zeros, which the step leaves zero)
        LaunchTimer t(c, KC_DESCENT);
        launch_descent(fuse->x + ly.b_off, g + ly.b_off, lo.d_pad, fuse->v + ly.b_off,
                       fuse->S + ly.b_off, fuse->y + ly.b_off, nullptr, nullptr, 0, lo.d_pad,
                       round_up(ly.out, 4), K, fuse->lam, fuse->lr, fuse->mu, fuse->nesterov, nullptr, s,
                       fuse->restart);
      }
    };
    auto input_grad = [&]() -> int {
      GemmDesc d{};
      d.b32s = bf;
      d.A = dz; d.strideA = astride(l + 1); d.ldA = ld_dz; d.a_kmajor = 1; d.cbA = b32s_blocks(ly.out);
      d.B = wptr(l); d.strideB = wstride; d.ldB = ly.ldw; d.b_kmajor = 0; d.cbB = b32s_blocks(ly.in);
      d.C = c->at<char>(lo.dz[l]); d.strideC = astride(l); d.ldC = lo.ld[l]; d.cbC = b32s_blocks(ly.in);
      d.M = B; d.N = ly.in; d.Kd = ly.out; d.batch = K;
      d.in_bf16 = bf; d.out_bf16 = bf; d.epilogue = EPI_MASK;
      d.mask = act; d.strideMask = astride(l); d.ldMask = lo.ld[l]; d.cbMask = b32s_blocks(ly.in);
      split(c, d);
      LaunchTimer t(c, KC_GEMM_DX);
      if (launch_gemm(d, s) != 0) return fail(LSAM_EINVAL, "dX GEMM of layer %d rejected", l);
      return LSAM_OK;
    };
    const bool want_dx = l > l0 || need_dA0;
    int rc = LSAM_OK;
    // With the fused step the weight-gradient kernel overwrites the operand copy of W_l that
    // the input gradient still has to read, so that one goes first.
    if (fuse && want_dx && (rc = input_grad()) != LSAM_OK) return rc;
    if ((rc = weight_grad()) != LSAM_OK) return rc;
    bias_grad();
    if (!fuse && want_dx && (rc = input_grad()) != LSAM_OK) return rc;
  }
  if (l0 > 0) {
    int rc = conv_backward(c, static_cast<const float*>(X), params, ssq, &slots);
    if (rc != LSAM_OK) return rc;
  }
  if (ssq) {
    if (slots > lo.nblk) return fail(LSAM_ESTATE, "gradient-norm partials overran their buffer");
    c->norm_slots = slots;
  }
  return check_launch("forward/backward");
}

// bf16 dense model with the fused step: the weight gradients of the first pass were only summed
// (their squares), not stored.  Now that the norm is known each is computed once more from the
// dZ_l and A_{l-1} the first pass left behind, and its epilogue writes the operand copy of the
// perturbed weights bf16(x + scale g1) directly: 6 bytes per parameter (x read, copy written)
// instead of the 14 of storing g1, reading it back with x and writing the copy, at the price of
// one more contraction per layer, which the matrix units have room for.  Biases need no copy:
// the second pass's GEMMs form x_b + scale g1_b from the stored bias gradient.
int ascend_pass(lsam_ctx* c, const void* A0) {
  const Layout& lo = c->lo;
  const int K = lo.K, B = lo.B, L = lo.L;
  auto width = [&](int l) { return l < L ? lo.layers[l].in : lo.layers[L - 1].out; };
  auto astride = [&](int l) { return lo.act_elems(width(l), lo.ld[l]); };
  for (int l = L - 1; l >= 0; --l) {
    const Layer& ly = lo.layers[l];
    GemmDesc d{};
    d.b32s = 1;
    d.A = c->at<char>(lo.dz[l + 1]); d.strideA = astride(l + 1); d.ldA = lo.ld[l + 1]; d.a_kmajor = 0;
    d.cbA = b32s_blocks(ly.out);
    d.B = l == 0 ? A0 : (const void*)c->at<char>(lo.act[l]); d.strideB = astride(l); d.ldB = lo.ld[l];
    d.b_kmajor = 0; d.cbB = b32s_blocks(ly.in);
    d.C = c->at<float>(lo.g) + ly.w_off; d.strideC = lo.d_pad; d.ldC = ly.ldw;
    d.M = ly.out; d.N = ly.in; d.Kd = B; d.batch = K;
    d.in_bf16 = 1; d.out_bf16 = 0; d.epilogue = EPI_PLAIN;
    AscentFusion f;
    f.x = c->at<float>(lo.x) + ly.w_off;
    f.scale = c->at<float>(lo.scale);
    f.shadow = c->at<uint16_t>(lo.xt) + lo.shadow_off[l];
    f.shadow_stride = lo.shadow_stride;
    f.cbShadow = b32s_blocks(ly.in);
    d.ascend = &f;
    LaunchTimer t(c, KC_GEMM_DW_ASCEND);
    if (launch_gemm(d, c->stream) != 0) return fail(LSAM_EINVAL, "ascent GEMM of layer %d rejected", l);
  }
  return check_launch("ascent GEMMs");
}

// Norm of g1 and the perturbed point.  `partials_ready`: the kernels that wrote g1 already
// left the partial sums of its squares.  With rho = 0 the perturbed point is x itself and is
// not written.
int update_tail_first(lsam_ctx* c, const float* g1, int64_t g_stride, int64_t n, float* loss,
                      bool partials_ready, bool perturb = true) {
  const Layout& lo = c->lo;
  hipStream_t s = c->stream;
  int nparts = partials_ready ? c->norm_slots : (lo.nblk < 1024 ? lo.nblk : 1024);
  if (!partials_ready) {
    LaunchTimer t(c, KC_SUMSQ);
    launch_sumsq_partials(g1, g_stride, n, lo.K, c->at<double>(lo.partials), nparts, s);
  }
  {
    LaunchTimer t(c, KC_NORM_FINISH);
    launch_norm_finish(c->at<double>(lo.partials), nparts, partials_ready ? lo.nblk : nparts, lo.K,
                       c->rho, c->cfg.gamma,
                       c->at<float>(lo.norms), c->at<float>(lo.scale),
                       lo.raw ? nullptr : c->at<float>(lo.loss_rows), lo.B,
                       lo.raw ? nullptr : (loss ? loss : c->at<float>(lo.loss)), s,
                       c->at<int32_t>(lo.restart));
  }
  if (c->rho != 0.f && perturb) {
    LaunchTimer t(c, KC_PERTURB);
    launch_perturb(c->at<float>(lo.x), g1, g_stride, c->at<float>(lo.scale),
                   lo.bf16 ? nullptr : c->at<float>(lo.xt),
                   lo.bf16 ? c->at<uint16_t>(lo.xt) : nullptr, &lo.map, lo.shadow_stride, lo.d_pad, n,
                   lo.K, s);
  }
  return check_launch("norm/perturb");
}

// Whether the sampler step of this configuration can ride in the epilogues of the second
// pass's weight-gradient GEMMs: bf16 dense model, Algorithm 2 (the data-parallel baseline needs
// the averaged gradient first), no Langevin noise.
bool can_fuse_step(const lsam_ctx* c) {
  return c->lo.bf16 && c->cfg.algorithm == LSAM_ALG_LSAM && !(c->cfg.noise_scale > 0.f) && c->fuse_step;
}

int update_tail_second(lsam_ctx* c, const float* g2, int64_t g_stride, int64_t n, bool already_stepped = false) {
  const Layout& lo = c->lo;
  if (already_stepped) {
    ++c->t_step;
    c->sched.tick();
    return check_launch("descent");
  }
  ReplicaScalars lam;
  for (int i = 0; i < lo.K; ++i) lam.v[i] = coupling(c, i);
  const NoiseMap* noise = nullptr;
  if (c->cfg.noise_scale > 0.f) {
    c->noise.step = c->t_step;
    c->noise.amp = (float)((double)c->cfg.noise_scale * std::sqrt(2.0 * (double)c->lr));
    noise = &c->noise;
  }
  {
    LaunchTimer t(c, KC_DESCENT);
    launch_descent(c->at<float>(lo.x), g2, g_stride, c->at<float>(lo.v), c->at<float>(lo.S),
                   c->at<float>(lo.y), lo.bf16 ? c->at<uint16_t>(lo.xt) : nullptr, &lo.map,
                   lo.shadow_stride, lo.d_pad, n, lo.K, lam, c->lr, c->cfg.momentum, c->cfg.nesterov,
                   noise, c->stream, c->at<int32_t>(lo.restart));
  }
  ++c->t_step;
  c->sched.tick();
  return check_launch("descent");
}

// Host <-> device transfers go through a pinned staging buffer owned by the context, in
// pieces of at most kStageBytes, each followed by a stream synchronisation: pageable-memory
// copies are left to no one else's staging (a strided device-to-host copy into fresh pageable
// memory was seen to return with a few words not yet written when run under the profiler).
constexpr size_t kStageBytes = 64u << 20;

int ensure_stage(lsam_ctx* c) {
  if (c->stage) return LSAM_OK;
  HIP_TRY(hipHostMalloc(&c->stage, kStageBytes, hipHostMallocDefault));
  return LSAM_OK;
}

int to_host(lsam_ctx* c, void* dst, const void* src_dev, size_t bytes) {
  int rc = ensure_stage(c);
  if (rc != LSAM_OK) return rc;
  char* d = static_cast<char*>(dst);
  const char* s = static_cast<const char*>(src_dev);
  for (size_t off = 0; off < bytes; off += kStageBytes) {
    const size_t n = std::min(kStageBytes, bytes - off);
    HIP_TRY(hipMemcpyAsync(c->stage, s + off, n, hipMemcpyDeviceToHost, c->stream));
    HIP_TRY(hipStreamSynchronize(c->stream));
    memcpy(d + off, c->stage, n);
  }
  return LSAM_OK;
}

int to_device(lsam_ctx* c, void* dst_dev, const void* src, size_t bytes) {
  int rc = ensure_stage(c);
  if (rc != LSAM_OK) return rc;
  char* d = static_cast<char*>(dst_dev);
  const char* s = static_cast<const char*>(src);
  for (size_t off = 0; off < bytes; off += kStageBytes) {
    const size_t n = std::min(kStageBytes, bytes - off);
    memcpy(c->stage, s + off, n);
    HIP_TRY(hipMemcpyAsync(d + off, c->stage, n, hipMemcpyHostToDevice, c->stream));
    HIP_TRY(hipStreamSynchronize(c->stream));
  }
  return LSAM_OK;
}

// Copies between the public flat layout (host) and one padded replica vector (device): the
// rows of W_l lose or gain their padding on the host side of the staging buffer.
int copy_in(lsam_ctx* c, const float* src_flat, float* dst_dev) {
  const Layout& lo = c->lo;
  if (lo.raw) return to_device(c, dst_dev, src_flat, (size_t)lo.d * 4);
  int rc = ensure_stage(c);
  if (rc != LSAM_OK) return rc;
  float* stage = static_cast<float*>(c->stage);
  for (const Piece& p : lo.pieces) {
    if (p.rows == 1) {
      if ((rc = to_device(c, dst_dev + p.off, src_flat + p.flat, (size_t)p.cols * 4)) != LSAM_OK) return rc;
      continue;
    }
    const int64_t rows_per = std::max<int64_t>(1, (int64_t)(kStageBytes / 4) / p.ld);
    for (int64_t r0 = 0; r0 < p.rows; r0 += rows_per) {
      const int64_t nr = std::min<int64_t>(rows_per, p.rows - r0);
      for (int64_t r = 0; r < nr; ++r) {
        memcpy(stage + r * p.ld, src_flat + p.flat + (r0 + r) * p.cols, (size_t)p.cols * 4);
        if (p.ld > p.cols) memset(stage + r * p.ld + p.cols, 0, (size_t)(p.ld - p.cols) * 4);
      }
      HIP_TRY(hipMemcpyAsync(dst_dev + p.off + r0 * p.ld, stage, (size_t)nr * p.ld * 4,
                             hipMemcpyHostToDevice, c->stream));
      HIP_TRY(hipStreamSynchronize(c->stream));
    }
  }
  return LSAM_OK;
}

int copy_out(lsam_ctx* c, const float* src_dev, float* dst_flat) {
  const Layout& lo = c->lo;
  if (lo.raw) return to_host(c, dst_flat, src_dev, (size_t)lo.d * 4);
  int rc = ensure_stage(c);
  if (rc != LSAM_OK) return rc;
  const float* stage = static_cast<const float*>(c->stage);
  for (const Piece& p : lo.pieces) {
    if (p.rows == 1) {
      if ((rc = to_host(c, dst_flat + p.flat, src_dev + p.off, (size_t)p.cols * 4)) != LSAM_OK) return rc;
      continue;
    }
    const int64_t rows_per = std::max<int64_t>(1, (int64_t)(kStageBytes / 4) / p.ld);
    for (int64_t r0 = 0; r0 < p.rows; r0 += rows_per) {
      const int64_t nr = std::min<int64_t>(rows_per, p.rows - r0);
      HIP_TRY(hipMemcpyAsync(c->stage, src_dev + p.off + r0 * p.ld, (size_t)nr * p.ld * 4,
                             hipMemcpyDeviceToHost, c->stream));
      HIP_TRY(hipStreamSynchronize(c->stream));
      for (int64_t r = 0; r < nr; ++r)
        memcpy(dst_flat + p.flat + (r0 + r) * p.cols, stage + r * p.ld, (size_t)p.cols * 4);
    }
  }
  return LSAM_OK;
}

}  // namespace

extern "C" {

const char* lsam_last_error(void) { return g_err.c_str(); }

int64_t lsam_num_params(const lsam_config* cfg) {
  if (check_config(cfg) != LSAM_OK) return -1;
  Layout lo;
  build_layout(*cfg, lo);
  return lo.d;
}

size_t lsam_workspace_bytes(const lsam_config* cfg) {
  if (check_config(cfg) != LSAM_OK) return 0;
  Layout lo;
  build_layout(*cfg, lo);
  return lo.total;
}

int lsam_schedule_replay(const lsam_config* cfg, int32_t n_ticks, int32_t* due_out,
                         int32_t* tau_out) {
  int rc = check_config(cfg);
  if (rc != LSAM_OK) return rc;
  if (n_ticks < 0 || (!due_out && !tau_out)) return fail(LSAM_EINVAL, "nothing to replay into");
  Schedule s;
  s.init(*cfg);
  for (int t = 0; t < n_ticks; ++t) {
    if (tau_out)
      for (int i = 0; i < cfg->K; ++i) tau_out[(int64_t)t * cfg->K + i] = s.tau()[i];
    s.tick();
    DueList d = s.due();
    if (due_out) {
      for (int i = 0; i < cfg->K; ++i) due_out[(int64_t)t * cfg->K + i] = 0;
      for (int j = 0; j < d.n; ++j) due_out[(int64_t)t * cfg->K + d.idx[j]] = 1;
    }
    if (d.n) s.served(d);
  }
  return LSAM_OK;
}

int lsam_init(const lsam_config* cfg, const float* init_params, int64_t n_init, void* workspace,
              size_t workspace_bytes, void* stream, lsam_ctx** out) {
  if (!out) return fail(LSAM_EINVAL, "out is NULL");
  *out = nullptr;
  int rc = check_config(cfg);
  if (rc != LSAM_OK) return rc;
  if (!init_params) return fail(LSAM_EINVAL, "init_params is NULL");
  if (!workspace) return fail(LSAM_EINVAL, "workspace is NULL");
  if (reinterpret_cast<uintptr_t>(workspace) & 255)
    return fail(LSAM_EINVAL, "workspace must be 256-byte aligned");
  lsam_ctx* c = new (std::nothrow) lsam_ctx();
  if (!c) return fail(LSAM_ENOMEM, "host allocation failed");
  c->cfg = *cfg;
  if (cfg->n_layers > 0) {
    c->dims.assign(cfg->dims, cfg->dims + cfg->n_layers + 1);
    c->cfg.dims = c->dims.data();
  } else {
    c->cfg.dims = nullptr;
  }
  if (cfg->tau) {
    c->tau_explicit.assign(cfg->tau, cfg->tau + cfg->K);
    c->cfg.tau = c->tau_explicit.data();
  }
  build_layout(c->cfg, c->lo);
  const Layout& lo = c->lo;
  if (n_init != lo.d && n_init != (int64_t)(lo.K + 1) * lo.d) {
    delete c;
    return fail(LSAM_EINVAL, "n_init=%lld must be d=%lld or (K+1)*d", (long long)n_init,
                (long long)lo.d);
  }
  if (workspace_bytes < lo.total) {
    delete c;
    return fail(LSAM_ENOMEM, "workspace holds %zu bytes, %zu needed", workspace_bytes, lo.total);
  }
  c->ws = static_cast<char*>(workspace);
  c->stream = static_cast<hipStream_t>(stream);
  {
    NoiseMap& nm = c->noise;
    nm.key0 = (uint32_t)(c->cfg.noise_seed & 0xFFFFFFFFu);
    nm.key1 = (uint32_t)(c->cfg.noise_seed >> 32);
    nm.raw_n = lo.raw ? lo.d : 0;
    nm.n = 0;
    nm.seg = nullptr;
  }
  c->lr = cfg->lr;
  c->rho = cfg->rho;
  c->sched.init(c->cfg);

  auto bail = [&](int code) {
    if (c->stage) (void)hipHostFree(c->stage);
    delete c;
    return code;
  };
  launch_fill_zero(c->ws, lo.total, c->stream);
  if (check_launch("zero fill") != LSAM_OK) return bail(LSAM_EHIP);
  if (hipStreamSynchronize(c->stream) != hipSuccess)
    return bail(fail(LSAM_EHIP, "stream synchronize failed during init"));
  if (lo.noise_segs) {
    // the noise generator's table: one run per parameter group, in the layout's order
    std::vector<NoiseSeg> segs;
    for (const Piece& p : lo.pieces)
      segs.push_back(NoiseSeg{p.off, p.off + (p.rows == 1 ? (int64_t)p.cols : (int64_t)p.rows * p.ld), p.ld,
                              p.cols, p.code, 0});
    if ((rc = to_device(c, c->at<char>(lo.noise_segs), segs.data(), segs.size() * sizeof(NoiseSeg))) != LSAM_OK)
      return bail(rc);
    c->noise.seg = c->at<NoiseSeg>(lo.noise_segs);
    c->noise.n = (int)segs.size();
  }
  float* x = c->at<float>(lo.x);
  float* y = c->at<float>(lo.y);
  if (n_init == lo.d) {
    if ((rc = copy_in(c, init_params, y)) != LSAM_OK) return bail(rc);
    launch_broadcast(y, x, lo.d_pad, lo.d_pad, lo.K, c->stream);
  } else {
    for (int i = 0; i < lo.K; ++i)
      if ((rc = copy_in(c, init_params + (int64_t)i * lo.d, x + (int64_t)i * lo.d_pad)) != LSAM_OK)
        return bail(rc);
    if ((rc = copy_in(c, init_params + (int64_t)lo.K * lo.d, y)) != LSAM_OK) return bail(rc);
  }
  if (lo.bf16)
    launch_shadow_refresh(x, c->at<uint16_t>(lo.xt), lo.map, lo.d_pad, lo.shadow_stride, lo.d_pad,
                          lo.K, c->stream);
  if (check_launch("parameter broadcast") != LSAM_OK) return bail(LSAM_EHIP);
  if (hipStreamSynchronize(c->stream) != hipSuccess)
    return bail(fail(LSAM_EHIP, "stream synchronize failed during init"));
  *out = c;
  return LSAM_OK;
}

int lsam_step(lsam_ctx* c, const void* X, const int32_t* labels, float* loss) {
  if (!c) return fail(LSAM_EINVAL, "ctx is NULL");
  if (c->lo.raw) return fail(LSAM_ESTATE, "lsam_step needs an MLP configuration");
  if (!X || !labels) return fail(LSAM_EINVAL, "X or labels is NULL");
  const Layout& lo = c->lo;
  const void* A0 = X;
  if (reinterpret_cast<uintptr_t>(X) & 15) return fail(LSAM_EINVAL, "X must be 16-byte aligned");
  if (lo.bf16) {
    LaunchTimer t(c, KC_MISC);     // the input joins the other bf16 tensors in the blocked layout
    launch_rowmajor_to_b32s(static_cast<const uint16_t*>(X), c->at<uint16_t>(lo.a0), lo.B,
                            lo.layers[0].in, lo.K, c->stream);
    A0 = c->at<char>(lo.a0);
  } else if (lo.need_a0) {
    LaunchTimer t(c, KC_MISC);
    launch_pad_rows(X, c->at<char>(lo.a0), (int64_t)lo.K * lo.B, lo.layers[0].in, lo.ld[0],
                    (int)lo.es(), c->stream);
    A0 = c->at<char>(lo.a0);
  }
  int rc;
  const bool dp = c->cfg.algorithm == LSAM_ALG_DATA_PARALLEL;
  float* g = c->at<float>(lo.g);
  // data-parallel baseline: every replica's gradient is replaced by the average over replicas
  auto average = [&]() {
    LaunchTimer t(c, KC_MISC);
    launch_grad_mean(g, lo.d_pad, g, lo.d_pad, lo.d_pad, lo.K, lo.K, c->stream);
  };
  const void* w1 = lo.bf16 ? (const void*)c->at<char>(lo.xt) : (const void*)c->at<char>(lo.x);
  // bf16 dense model, Algorithm 2, no noise: neither gradient of a weight matrix is stored.
  // First pass: sums of squares only; then the ascent GEMMs; second pass: the sampler step in
  // the weight-gradient epilogues.
  const bool fused = c->rho != 0.f && can_fuse_step(c);
  if ((rc = forward_backward(c, A0, labels, w1, false, !dp, nullptr, fused)) != LSAM_OK) return rc;
  if (dp) average();
  if ((rc = update_tail_first(c, g, lo.d_pad, lo.d_pad, loss, !dp, !fused)) != LSAM_OK) return rc;
  if (fused && (rc = ascend_pass(c, A0)) != LSAM_OK) return rc;
  bool stepped = false;
  if (c->rho != 0.f) {     // otherwise the perturbed point is x and g already is its gradient
    SamplerFusion f;
    if (fused) {
      f.x = c->at<float>(lo.x); f.v = c->at<float>(lo.v); f.S = c->at<float>(lo.S);
      f.restart = c->at<int32_t>(lo.restart);
      f.y = c->at<float>(lo.y);
      f.shadow = c->at<uint16_t>(lo.xt); f.shadow_stride = lo.shadow_stride; f.cbShadow = 0;
      for (int i = 0; i < lo.K; ++i) f.lam.v[i] = coupling(c, i);
      f.lr = c->lr; f.mu = c->cfg.momentum; f.nesterov = c->cfg.nesterov;
      stepped = true;
    }
    if ((rc = forward_backward(c, A0, labels, c->at<char>(lo.xt), true, false, stepped ? &f : nullptr)) != LSAM_OK)
      return rc;
    if (dp) average();
  }
  return update_tail_second(c, g, lo.d_pad, lo.d_pad, stepped);
}

int lsam_step_grads(lsam_ctx* c, const float* g1, const float* g2) {
  if (!c) return fail(LSAM_EINVAL, "ctx is NULL");
  if (!c->lo.raw) return fail(LSAM_ESTATE, "lsam_step_grads needs raw-vector mode");
  if (!g1 || !g2) return fail(LSAM_EINVAL, "g1 or g2 is NULL");
  if ((reinterpret_cast<uintptr_t>(g1) & 3) || (reinterpret_cast<uintptr_t>(g2) & 3))
    return fail(LSAM_EINVAL, "gradients must be 4-byte aligned");
  int rc;
  const Layout& lo = c->lo;
  if (c->cfg.algorithm == LSAM_ALG_DATA_PARALLEL) {
    // one averaged vector, read by every replica (row stride 0)
    float* m = c->at<float>(lo.gmean);
    {
      LaunchTimer t(c, KC_MISC);
      launch_grad_mean(g1, lo.d, m, 0, lo.d, lo.K, 1, c->stream);
    }
    if ((rc = update_tail_first(c, m, 0, lo.d, nullptr, false)) != LSAM_OK) return rc;
    {
      LaunchTimer t(c, KC_MISC);
      launch_grad_mean(g2, lo.d, m, 0, lo.d, lo.K, 1, c->stream);
    }
    return update_tail_second(c, m, 0, lo.d);
  }
  if ((rc = update_tail_first(c, g1, lo.d, lo.d, nullptr, false)) != LSAM_OK) return rc;
  return update_tail_second(c, g2, lo.d, lo.d);
}

int lsam_sync(lsam_ctx* c) {
  if (!c) return fail(LSAM_EINVAL, "ctx is NULL");
  if (c->cfg.algorithm == LSAM_ALG_DATA_PARALLEL) return 0;   // no center in that baseline
  const Layout& lo = c->lo;
  const DueList due = c->sched.due();
  if (due.n == 0) return 0;
  const int64_t m = c->sched.samples(due);
  {
    LaunchTimer t(c, KC_CENTER);
    launch_center(c->at<float>(lo.S), c->at<float>(lo.y), c->at<float>(lo.gprev), lo.d_pad,
                  lo.raw ? lo.d : lo.d_pad, due, (float)(1.0 / (double)m), c->cfg.beta,
                  c->cfg.lr_center, c->sched.t_y() > 0 ? 1 : 0, c->stream, c->at<int32_t>(lo.restart));
  }
  int rc = check_launch("center update");
  if (rc != LSAM_OK) return rc;
  c->sched.served(due);
  return due.n;
}

int lsam_get_buffer(lsam_ctx* c, int32_t which, int32_t replica, float* dst, int64_t n) {
  if (!c || !dst) return fail(LSAM_EINVAL, "ctx or dst is NULL");
  const Layout& lo = c->lo;
  if (n != lo.d) return fail(LSAM_EINVAL, "n=%lld must equal d=%lld", (long long)n, (long long)lo.d);
  if (replica < -1 || replica >= lo.K) return fail(LSAM_EINVAL, "replica %d out of range", replica);
  HIP_TRY(hipStreamSynchronize(c->stream));
  const int64_t roff = (int64_t)(replica < 0 ? 0 : replica) * lo.d_pad;
  switch (which) {
    case LSAM_BUF_PARAMS:
      return copy_out(c, replica < 0 ? c->at<float>(lo.y) : c->at<float>(lo.x) + roff, dst);
    case LSAM_BUF_CENTER_DIR:
      return copy_out(c, c->at<float>(lo.gprev), dst);
    default: break;
  }
  if (replica < 0) return fail(LSAM_EINVAL, "replica -1 is valid for the parameters only");
  switch (which) {
    case LSAM_BUF_VELOCITY: return copy_out(c, c->at<float>(lo.v) + roff, dst);
    case LSAM_BUF_ITER_SUM: {
      // a sum the last center update served reads as zero; its memory is rewritten by the next step
      int32_t mark = 0;
      int rc = to_host(c, &mark, c->at<int32_t>(lo.restart) + replica, 4);
      if (rc != LSAM_OK) return rc;
      if (mark == 2) {
        memset(dst, 0, (size_t)n * 4);
        return LSAM_OK;
      }
      return copy_out(c, c->at<float>(lo.S) + roff, dst);
    }
    case LSAM_BUF_GRAD:
      if (lo.raw) return fail(LSAM_ESTATE, "raw-vector mode keeps no gradient buffer");
      return copy_out(c, c->at<float>(lo.g) + roff, dst);
    case LSAM_BUF_PERTURBED: {
      if (!lo.bf16) return copy_out(c, c->at<float>(lo.xt) + roff, dst);
      // bf16 operand copy of the weight matrices: fetch this replica's copy, widen and undo
      // the blocked layout on the host; biases are not part of the copy (the GEMMs read the
      // fp32 ones), they are reported from the master parameters
      std::vector<uint16_t> h((size_t)lo.shadow_stride);
      int rc0 = to_host(c, h.data(), c->at<uint16_t>(lo.xt) + (int64_t)replica * lo.shadow_stride,
                        (size_t)lo.shadow_stride * 2);
      if (rc0 != LSAM_OK) return rc0;
      int rc = copy_out(c, c->at<float>(lo.x) + roff, dst);
      if (rc != LSAM_OK) return rc;
      for (int l = 0; l < lo.L; ++l) {
        const Layer& ly = lo.layers[l];
        const int cb = b32s_blocks(ly.in);
        for (int r = 0; r < ly.out; ++r)
          for (int q = 0; q < ly.in; ++q) {
            const uint32_t u = (uint32_t)h[(size_t)(lo.shadow_off[l] + b32s_offset(r, q, cb))] << 16;
            float f;
            memcpy(&f, &u, 4);
            dst[ly.w_flat + (int64_t)r * ly.in + q] = f;
          }
      }
      return LSAM_OK;
    }
    default: return fail(LSAM_EINVAL, "unknown buffer id %d", which);
  }
}

int lsam_set_buffer(lsam_ctx* c, int32_t which, int32_t replica, const float* src, int64_t n) {
  if (!c || !src) return fail(LSAM_EINVAL, "ctx or src is NULL");
  const Layout& lo = c->lo;
  if (n != lo.d) return fail(LSAM_EINVAL, "n=%lld must equal d=%lld", (long long)n, (long long)lo.d);
  if (replica < -1 || replica >= lo.K) return fail(LSAM_EINVAL, "replica %d out of range", replica);
  HIP_TRY(hipStreamSynchronize(c->stream));
  const int64_t roff = (int64_t)(replica < 0 ? 0 : replica) * lo.d_pad;
  float* dst = nullptr;
  switch (which) {
    case LSAM_BUF_PARAMS: dst = replica < 0 ? c->at<float>(lo.y) : c->at<float>(lo.x) + roff; break;
    case LSAM_BUF_CENTER_DIR: dst = c->at<float>(lo.gprev); break;
    case LSAM_BUF_VELOCITY: dst = replica < 0 ? nullptr : c->at<float>(lo.v) + roff; break;
    case LSAM_BUF_ITER_SUM: dst = replica < 0 ? nullptr : c->at<float>(lo.S) + roff; break;
    default: return fail(LSAM_EINVAL, "buffer id %d cannot be set", which);
  }
  if (!dst) return fail(LSAM_EINVAL, "replica -1 is valid for the parameters only");
  int rc = copy_in(c, src, dst);
  if (rc != LSAM_OK) return rc;
  if (which == LSAM_BUF_ITER_SUM) {
    // the sum is what the caller wrote from now on, not "zero since the last center update"
    const int32_t none = 0;
    if ((rc = to_device(c, c->at<int32_t>(lo.restart) + replica, &none, 4)) != LSAM_OK) return rc;
  }
  if (which == LSAM_BUF_PARAMS && replica >= 0 && lo.bf16) {
    launch_shadow_refresh(dst, c->at<uint16_t>(lo.xt) + (int64_t)replica * lo.shadow_stride, lo.map,
                          lo.d_pad, lo.shadow_stride, lo.d_pad, 1, c->stream);
    if ((rc = check_launch("bf16 operand refresh")) != LSAM_OK) return rc;
    HIP_TRY(hipStreamSynchronize(c->stream));
  }
  return LSAM_OK;
}

int lsam_get_params(lsam_ctx* c, int32_t replica, float* dst, int64_t n) {
  return lsam_get_buffer(c, LSAM_BUF_PARAMS, replica, dst, n);
}

int lsam_get_norms(lsam_ctx* c, float* dst) {
  if (!c || !dst) return fail(LSAM_EINVAL, "ctx or dst is NULL");
  HIP_TRY(hipStreamSynchronize(c->stream));
  {
    int rc0 = to_host(c, dst, c->at<float>(c->lo.norms), (size_t)c->lo.K * 4);
    if (rc0 != LSAM_OK) return rc0;
  }
  return LSAM_OK;
}

int lsam_get_schedule(lsam_ctx* c, int32_t* tau_out, int32_t* count_out, int64_t* t_y_out) {
  if (!c) return fail(LSAM_EINVAL, "ctx is NULL");
  for (int i = 0; i < c->lo.K; ++i) {
    if (tau_out) tau_out[i] = c->sched.tau()[i];
    if (count_out) count_out[i] = c->sched.count()[i];
  }
  if (t_y_out) *t_y_out = c->sched.t_y();
  return LSAM_OK;
}

int lsam_layer_info(lsam_ctx* c, int32_t layer, int32_t* info, int32_t n) {
  if (!c || !info) return fail(LSAM_EINVAL, "ctx or info is NULL");
  const Layout& lo = c->lo;
  if (lo.raw) return fail(LSAM_ESTATE, "raw-vector mode has no layers");
  if (layer < 0 || layer >= lo.L) return fail(LSAM_EINVAL, "layer %d out of range 0..%d", layer, lo.L - 1);
  if (n < LSAM_LAYER_INFO_FIELDS) return fail(LSAM_EINVAL, "info needs %d entries", LSAM_LAYER_INFO_FIELDS);
  const Layer& ly = lo.layers[layer];
  int kind = LSAM_LAYER_DENSE, dx_stored = 0;
  int64_t rows = lo.B;
  if (layer < lo.n_conv) {
    const ConvLayer& cv = lo.conv[layer];
    kind = cv.first ? LSAM_LAYER_CONV_FIRST : cv.direct_in ? LSAM_LAYER_CONV_DIRECT : LSAM_LAYER_CONV_STORED;
    dx_stored = (layer > 0 && !cv.direct_dx) ? 1 : 0;
    rows = cv.rows;
  } else if (layer == lo.L - 1 && head_is_fused(lo)) {
    kind = LSAM_LAYER_HEAD;
  }
  const bool fused = c->rho != 0.f && can_fuse_step(c);
  info[0] = kind;
  info[1] = dx_stored;
  info[2] = fused ? (gram_norm_pays(lo.B, ly.out, ly.in) ? 2 : 1) : 0;
  info[3] = (int32_t)rows;
  info[4] = ly.in;
  info[5] = ly.out;
  info[6] = ly.proj ? ly.proj_in : 0;
  info[7] = ly.proj ? lo.conv[layer].skip_step : 0;
  return LSAM_OK;
}

int lsam_set_fused_step(lsam_ctx* c, int32_t on) {
  if (!c) return fail(LSAM_EINVAL, "ctx is NULL");
  c->fuse_step = on != 0;
  return can_fuse_step(c) ? 1 : 0;
}

int lsam_note_replay(lsam_ctx* c) {
  if (!c) return fail(LSAM_EINVAL, "ctx is NULL");
  // a captured step carries the kernel arguments of the step it was captured from: the coupling
  // coefficients lambda0/(lr tau_i) and the noise counter are frozen in the graph
  if (c->cfg.noise_scale > 0.f)
    return fail(LSAM_ESTATE, "a replayed step would repeat its Langevin noise");
  if (c->cfg.sched_mode == LSAM_SCHED_REDRAW && !c->cfg.tau && c->cfg.lambda_abs < 0.f &&
      c->cfg.algorithm == LSAM_ALG_LSAM)
    return fail(LSAM_ESTATE, "redrawn periods change lambda_i, which a replayed step cannot follow");
  ++c->t_step;
  c->sched.tick();
  return LSAM_OK;
}

int lsam_get_counters(lsam_ctx* c, int64_t* state, int64_t n) {
  if (!c || !state) return fail(LSAM_EINVAL, "ctx or state is NULL");
  const int K = c->lo.K;
  if (n != 2 * (int64_t)K + 3) return fail(LSAM_EINVAL, "n=%lld must equal 2K+3=%d", (long long)n, 2 * K + 3);
  for (int i = 0; i < K; ++i) {
    state[i] = c->sched.count()[i];
    state[K + i] = c->sched.tau()[i];
  }
  state[2 * K] = (int64_t)c->sched.generator_state();
  state[2 * K + 1] = c->sched.t_y();
  state[2 * K + 2] = (int64_t)c->t_step;
  return LSAM_OK;
}

int lsam_set_counters(lsam_ctx* c, const int64_t* state, int64_t n) {
  if (!c || !state) return fail(LSAM_EINVAL, "ctx or state is NULL");
  const int K = c->lo.K;
  if (n != 2 * (int64_t)K + 3) return fail(LSAM_EINVAL, "n=%lld must equal 2K+3=%d", (long long)n, 2 * K + 3);
  if (state[2 * K + 2] < 0 || state[2 * K + 2] > (int64_t)UINT32_MAX)
    return fail(LSAM_EINVAL, "noise step %lld out of range", (long long)state[2 * K + 2]);
  if (!c->sched.restore(state, state + K, (uint64_t)state[2 * K], state[2 * K + 1]))
    return fail(LSAM_EINVAL, "counts must be >= 0, periods >= 1, the sync count >= 0");
  c->t_step = (uint32_t)state[2 * K + 2];
  return LSAM_OK;
}

int lsam_get_activation(lsam_ctx* c, int32_t layer, int32_t replica, float* dst, int64_t n) {
  if (!c || !dst) return fail(LSAM_EINVAL, "ctx or dst is NULL");
  const Layout& lo = c->lo;
  if (lo.raw || lo.n_conv > 0) return fail(LSAM_ESTATE, "activations can be read from a dense model only");
  if (layer < 1 || layer >= lo.L) return fail(LSAM_EINVAL, "layer %d is not a hidden layer (1..%d)", layer, lo.L - 1);
  if (replica < 0 || replica >= lo.K) return fail(LSAM_EINVAL, "replica %d out of range", replica);
  const int width = lo.layers[layer].in, B = lo.B;
  if (n != (int64_t)B * width)
    return fail(LSAM_EINVAL, "n=%lld must equal batch*width=%lld", (long long)n, (long long)B * width);
  HIP_TRY(hipStreamSynchronize(c->stream));
  const int64_t elems = lo.act_elems(width, lo.ld[layer]);
  if (!lo.bf16) {
    std::vector<float> h((size_t)elems);
    int rc = to_host(c, h.data(), c->at<float>(lo.act[layer]) + (int64_t)replica * elems, (size_t)elems * 4);
    if (rc != LSAM_OK) return rc;
    for (int b = 0; b < B; ++b)
      memcpy(dst + (int64_t)b * width, h.data() + (int64_t)b * lo.ld[layer], (size_t)width * 4);
    return LSAM_OK;
  }
  std::vector<uint16_t> h((size_t)elems);
  int rc = to_host(c, h.data(), c->at<uint16_t>(lo.act[layer]) + (int64_t)replica * elems, (size_t)elems * 2);
  if (rc != LSAM_OK) return rc;
  const int cb = b32s_blocks(width);
  for (int b = 0; b < B; ++b)
    for (int q = 0; q < width; ++q) {
      const uint32_t u = (uint32_t)h[(size_t)b32s_offset(b, q, cb)] << 16;
      memcpy(dst + (int64_t)b * width + q, &u, 4);
    }
  return LSAM_OK;
}

int lsam_set_scalars(lsam_ctx* c, float lr, float rho) {
  if (!c) return fail(LSAM_EINVAL, "ctx is NULL");
  if (!(rho >= 0.f) || !(lr >= 0.f)) return fail(LSAM_EINVAL, "lr and rho must be >= 0");
  if (!(lr > 0.f) && c->cfg.lambda_abs < 0.f)
    return fail(LSAM_EINVAL, "lr must be > 0 when lambda is derived as lambda0/(lr*tau)");
  c->lr = lr;
  c->rho = rho;
  return LSAM_OK;
}

int lsam_timing_enable(lsam_ctx* c, int32_t on) {
  if (!c) return fail(LSAM_EINVAL, "ctx is NULL");
  int rc = drain_timing(c);
  if (rc != LSAM_OK) return rc;
  c->timing = on != 0;
  if (!on) {
    for (int i = 0; i < KC_COUNT; ++i) { c->t_count[i] = 0; c->t_ms[i] = 0.0; }
  }
  return LSAM_OK;
}

int lsam_timing_read(lsam_ctx* c, int32_t cap, const char** names, int64_t* counts,
                     double* total_ms) {
  if (!c || !names || !counts || !total_ms) return fail(LSAM_EINVAL, "NULL argument");
  int rc = drain_timing(c);
  if (rc != LSAM_OK) return rc;
  int n = 0;
  for (int i = 0; i < KC_COUNT && n < cap; ++i) {
    names[n] = kClassNames[i];
    counts[n] = c->t_count[i];
    total_ms[n] = c->t_ms[i];
    ++n;
  }
  return n;
}

int lsam_probe_peaks(void* scratch, size_t scratch_bytes, void* stream, double* copy_gbytes_per_s,
                     double* mfma_bf16_tflops, double* mfma_fp32_tflops) {
  if (!scratch || !copy_gbytes_per_s || !mfma_bf16_tflops || !mfma_fp32_tflops)
    return fail(LSAM_EINVAL, "NULL argument");
  if (scratch_bytes < 32768 || (reinterpret_cast<uintptr_t>(scratch) & 15))
    return fail(LSAM_EINVAL, "scratch must be 16-byte aligned and hold at least 32 KiB");
  if (probe_peaks(scratch, scratch_bytes, static_cast<hipStream_t>(stream), copy_gbytes_per_s,
                  mfma_bf16_tflops, mfma_fp32_tflops) != 0)
    return fail(LSAM_EHIP, "peak probe failed: %s", hipGetErrorString(hipGetLastError()));
  return LSAM_OK;
}

void lsam_destroy(lsam_ctx* c) {
  if (!c) return;
  (void)hipStreamSynchronize(c->stream);
  for (auto& t : c->pending) { (void)hipEventDestroy(t.a); (void)hipEventDestroy(t.b); }
  for (auto e : c->free_events) (void)hipEventDestroy(e);
  if (c->stage) (void)hipHostFree(c->stage);
  delete c;
}

}  // extern "C"
