// Log-masses of the text key blocks (paper Sec. 3.2, Sec. 4.1; Alg. 1 steps 5-7):
//   Lmass[n][N+i] = log sum_{t in text block i} exp(scale * q^pool_n . k_t)
// as a device function, because two launches carry it: text_mass_kernel by itself, and the launch
// that pools V (the streaming of V is bound by HBM, this by the vector ALU).
#pragma once
#include "rsa_common.hpp"

namespace rsa {

constexpr int kTextMassQueries = 8;                                   // pooled queries per workgroup
template <int D>
constexpr int text_mass_lds_floats() { return kTextMassQueries * D + kTextMassQueries * 256; }

__device__ inline float text_wave_max(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o));
  return v;
}
__device__ inline float text_wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
  return v;
}

// Eight pooled queries (n0 .. n0 + 7 of (batch, head) bh) against the individual text keys, 256 tokens
// at a time (a multiple of the block size), then one log-sum-exp per (query, text block). 256 threads;
// `lds`: text_mass_lds_floats<D>() floats.
template <int D, int BLK>
__device__ __forceinline__ void text_mass_block(const Dims& dm, const ScoreArgs& a, int n0, int bh, float* lds) {
  constexpr int NQ = kTextMassQueries;
  float (*qs)[D] = reinterpret_cast<float (*)[D]>(lds);
  float (*u)[256] = reinterpret_cast<float (*)[256]>(lds + NQ * D);
  const int b = bh / dm.heads, h = bh % dm.heads;
  const float* Qp = a.Qp + (size_t)bh * dm.n * D;
  for (int idx = threadIdx.x; idx < NQ * D; idx += 256) {
    const int r = idx / D, c = idx % D;
    qs[r][c] = (n0 + r < dm.n) ? Qp[(size_t)(n0 + r) * D + c] : 0.f;
  }
  __syncthreads();
  const uint16_t* Kt = a.K + (int64_t)b * dm.sb + (int64_t)h * dm.sh + dm.tv * dm.st;
  float* L = a.Lmass + (size_t)bh * dm.n * dm.m;
  const int wave = threadIdx.x / 64, lane = threadIdx.x % 64;

  for (int64_t c0 = 0; c0 < dm.tt; c0 += 256) {
    const int64_t tok = c0 + threadIdx.x;
    float acc[NQ];
#pragma unroll
    for (int r = 0; r < NQ; ++r) acc[r] = 0.f;
    if (tok < dm.tt) {
      const uint4* row = reinterpret_cast<const uint4*>(Kt + tok * dm.st);
#pragma unroll 4
      for (int cc = 0; cc < D / 8; ++cc) {
        const uint4 v = row[cc];
        const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const float k0 = bf16_bits_to_float(w[i] & 0xffffu), k1 = bf16_bits_to_float(w[i] >> 16);
#pragma unroll
          for (int r = 0; r < NQ; ++r) {
            acc[r] = fmaf(qs[r][cc * 8 + 2 * i], k0, acc[r]);
            acc[r] = fmaf(qs[r][cc * 8 + 2 * i + 1], k1, acc[r]);
          }
        }
      }
    }
#pragma unroll
    for (int r = 0; r < NQ; ++r) u[r][threadIdx.x] = acc[r] * dm.scale;
    __syncthreads();
    // tasks: (query r, block j of this chunk); one wave per task
    constexpr int BPC = 256 / BLK;
    for (int task = wave; task < NQ * BPC; task += 4) {
      const int r = task / BPC, j = task % BPC;
      const int64_t first = c0 + (int64_t)j * BLK;
      if (first >= dm.tt || n0 + r >= dm.n) continue;
      const int cnt = (int)((dm.tt - first) < BLK ? (dm.tt - first) : BLK);
      float mx = -INFINITY;
      for (int i = lane; i < cnt; i += 64) mx = fmaxf(mx, u[r][j * BLK + i]);
      mx = text_wave_max(mx);
      float sum = 0.f;
      for (int i = lane; i < cnt; i += 64) sum += expf(u[r][j * BLK + i] - mx);
      sum = text_wave_sum(sum);
      if (lane == 0) L[(size_t)(n0 + r) * dm.m + dm.n + (int)(first / BLK)] = mx + logf(sum);
    }
    __syncthreads();
  }
}

}  // namespace rsa
