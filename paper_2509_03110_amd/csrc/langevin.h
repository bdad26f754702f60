// Langevin noise of the sampler (Section "Langevin Dynamics for Sampling": SGLD as the Sampler
// of Algorithm 2):  x <- x - eta (G + mu v) + sigma sqrt(2 eta) xi,  xi ~ N(0, I).
//
// xi comes from Philox4x32-10 (Salmon, Moraes, Dror, Shaw, SC'11), a counter-based generator:
// the four normals of four neighbouring columns are a function of where they are and when,
//   counter = (column / 4, row, (8 * layer + piece) | replica << 16, step)        layered models
//   counter = (j / 4 mod 2^32, j / 4 >> 32, replica << 16, step)                  raw vector
//   piece: 0 W, 1 b, 2 gamma, 3 beta of the layer; 4..7 the same four of its projection shortcut
//   key     = (seed mod 2^32, seed >> 32)
//   u_i = ((r_i >> 8) + 1/2) / 2^24;  z0, z1 = sqrt(-2 ln u0) (cos, sin)(2 pi u1);  z2, z3 from u2, u3
// (a vector counts as one row), so no generator state is stored and the kernel that
// streams the parameters produces the noise on the way.
#pragma once
#include <stdint.h>

#include "../../include/lsam.h"

namespace lsam {

// One run of the padded flat layout that takes noise: a matrix (rows of `ld` floats, the first
// `cols` of each real) or a vector (one row).
struct NoiseSeg {
  int64_t begin, end;     // flat offsets inside a replica
  int32_t ld, cols;
  int32_t code;           // 8 * layer + piece
  int32_t pad_;
};
struct NoiseMap {
  int32_t n;                              // 0: raw vector of `raw_n` elements
  uint32_t key0, key1, step;
  float amp;                              // sigma * sqrt(2 eta)
  int64_t raw_n;
  const NoiseSeg* seg;                    // device memory, n runs in increasing order of `begin`
};
struct NoNoise {};

__device__ inline void philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3,
                                     uint32_t k0, uint32_t k1, uint32_t (&out)[4]) {
#pragma unroll
  for (int r = 0; r < 10; ++r) {
    const uint32_t hi0 = __umulhi(0xD2511F53u, c0), lo0 = 0xD2511F53u * c0;
    const uint32_t hi1 = __umulhi(0xCD9E8D57u, c2), lo1 = 0xCD9E8D57u * c2;
    c0 = hi1 ^ c1 ^ k0;
    c1 = lo1;
    c2 = hi0 ^ c3 ^ k1;
    c3 = lo0;
    k0 += 0x9E3779B9u;
    k1 += 0xBB67AE85u;
  }
  out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

__device__ inline void normals4(const uint32_t (&r)[4], float (&z)[4]) {
#pragma unroll
  for (int p = 0; p < 2; ++p) {
    const float u0 = ((float)(r[2 * p] >> 8) + 0.5f) * (1.0f / 16777216.0f);
    const float u1 = ((float)(r[2 * p + 1] >> 8) + 0.5f) * (1.0f / 16777216.0f);
    const float rad = sqrtf(-2.0f * logf(u0));
    float sn, cs;
    sincospif(2.0f * u1, &sn, &cs);
    z[2 * p] = rad * cs;
    z[2 * p + 1] = rad * sn;
  }
}

// amp * xi for the 4 elements at padded flat offset `flat` (a multiple of 4) of `replica`;
// zero for padding.  Rows are 8-aligned in the flat layout, so the 4 elements share a row and
// a column group.
__device__ inline void langevin4(const NoiseMap& m, int replica, int64_t flat, float (&out)[4]) {
  out[0] = out[1] = out[2] = out[3] = 0.f;
  uint32_t c0, c1, c2;
  int valid = 4;
  if (m.n == 0) {
    if (flat >= m.raw_n) return;
    const uint64_t grp = (uint64_t)flat >> 2;
    c0 = (uint32_t)grp; c1 = (uint32_t)(grp >> 32); c2 = (uint32_t)replica << 16;
    if (m.raw_n - flat < 4) valid = (int)(m.raw_n - flat);
  } else {
    // the last run that begins at or before `flat`
    int lo = 0, hi = m.n;
    while (hi - lo > 1) {
      const int mid = (lo + hi) >> 1;
      if (m.seg[mid].begin <= flat) lo = mid; else hi = mid;
    }
    const NoiseSeg sg = m.seg[lo];
    if (flat < sg.begin || flat >= sg.end) return;
    const uint32_t rel = (uint32_t)(flat - sg.begin);
    const uint32_t row = rel / (uint32_t)sg.ld;
    const uint32_t col = rel - row * (uint32_t)sg.ld;
    if ((int)col >= sg.cols) return;
    if (sg.cols - (int)col < 4) valid = sg.cols - (int)col;
    c0 = col >> 2; c1 = row; c2 = (uint32_t)sg.code | ((uint32_t)replica << 16);
  }
  uint32_t r[4];
  float z[4];
  philox4x32_10(c0, c1, c2, m.step, m.key0, m.key1, r);
  normals4(r, z);
#pragma unroll
  for (int e = 0; e < 4; ++e) out[e] = e < valid ? m.amp * z[e] : 0.f;
}

}  // namespace lsam
