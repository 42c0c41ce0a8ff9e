// Implicit full attention from pooled query-key interactions (paper Sec. 3.2, Sec. 4.1;
// Alg. 1 steps 5-7). Everything stays fp32: the selection that follows compares these
// values and is checked against an fp64 reference inside a 1e-4 band.
//
//   pooled_scores_kernel   Spool[n][m] = scale * q^pool_n . k^pool_m       (N x M x d, tiny)
//   text_mass_kernel       Lmass[n][N+i] = log sum_{t in text block i} exp(scale * q^pool_n . k_t)
//   ipar_softmax_rows_kernel  Lmass[n][m<N] = Spool + ln c_m ; Apool = row-softmax(Lmass)
//
// softmax(Lmass) is the paper's reallocation written in log space: the mixed softmax
// over [pooled video keys ; text tokens] gives weights proportional to exp(score); a video
// block is then multiplied by its token count (exp(s + ln c)), text tokens are summed per
// block (exp(logsumexp)), and everything is divided by the row total.
#include "rsa_common.hpp"

namespace rsa {
namespace {

__device__ inline float wave_max(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o));
  return v;
}
__device__ inline float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
  return v;
}

// One wave per 32 x 32 output tile, v_mfma_f32_32x32x2_f32: fp32 operands, fp32 products and
// sums, so the scores keep full single precision (the selection that follows is compared with
// fp64 inside a 1e-4 band). The contraction index may be visited in any order as long as both
// operands agree: k-step s takes channel s from the lanes of the lower half-wave and channel
// D/2 + s from the upper one, so every lane needs D/2 consecutive floats of its row.
// The 64 query rows and 64 key rows of a workgroup come in through LDS: read from global memory
// with every wave load covering two whole rows (a lane reading its own row directly touches 64
// cache lines per load and the kernel is then bound by the address unit of the CU), then read
// back per lane; a row stride of D + 4 floats keeps the 16-byte LDS reads free of bank conflicts.
template <int D>
__global__ __launch_bounds__(256) void pooled_scores_kernel(Dims dm, ScoreArgs a) {
  constexpr int KH = D / 2;                     // k-steps; channels per half-wave
  constexpr int RS = D + 4;                     // LDS row stride in floats
  constexpr int C4 = D / 4;                     // float4 per row
  __shared__ float rows[2][64 * RS];            // [0]: pooled queries n0 .. n0+63, [1]: pooled keys m0 .. m0+63
  const int bh = blockIdx.z;
  const int wave = threadIdx.x / 64, lane = threadIdx.x % 64;
  const int l32 = lane % 32, hf = lane / 32;
  const int nb = blockIdx.y * 64, mb = blockIdx.x * 64;
  for (int idx = threadIdx.x; idx < 64 * C4; idx += 256) {
    const int r = idx / C4, c4 = idx % C4;
    const int n = nb + r < dm.n ? nb + r : dm.n - 1;          // rows past the end repeat the last one (not stored)
    const int m = mb + r < dm.m ? mb + r : dm.m - 1;
    *reinterpret_cast<floatx4*>(&rows[0][r * RS + 4 * c4]) =
        *reinterpret_cast<const floatx4*>(a.Qp + ((size_t)bh * dm.n + n) * D + 4 * c4);
    *reinterpret_cast<floatx4*>(&rows[1][r * RS + 4 * c4]) =
        *reinterpret_cast<const floatx4*>(a.Kp + ((size_t)bh * dm.m + m) * D + 4 * c4);
  }
  __syncthreads();
  const int n0 = nb + (wave / 2) * 32, m0 = mb + (wave % 2) * 32;
  if (n0 >= dm.n || m0 >= dm.m) return;         // after the only barrier
  const floatx4* qrow = reinterpret_cast<const floatx4*>(&rows[0][((wave / 2) * 32 + l32) * RS + hf * KH]);
  const floatx4* krow = reinterpret_cast<const floatx4*>(&rows[1][((wave % 2) * 32 + l32) * RS + hf * KH]);
  floatx4 qv[KH / 4], kv[KH / 4];
#pragma unroll
  for (int i = 0; i < KH / 4; ++i) {
    qv[i] = qrow[i];
    kv[i] = krow[i];
  }
  floatx16 acc;
#pragma unroll
  for (int r = 0; r < 16; ++r) acc[r] = 0.f;
  // A = pooled queries (M = query row), B = pooled keys (N = key column)
#pragma unroll
  for (int i = 0; i < KH / 4; ++i)
#pragma unroll
    for (int e = 0; e < 4; ++e) acc = __builtin_amdgcn_mfma_f32_32x32x2f32(qv[i][e], kv[i][e], acc, 0, 0, 0);
  // accumulator register r: query row n0 + 8(r/4) + 4*hf + r%4, key column m0 + l32
  float* S = a.Spool + (size_t)bh * dm.n * dm.m;
  if (m0 + l32 < dm.m) {
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const int row = n0 + 8 * (r / 4) + 4 * hf + (r % 4);
      if (row < dm.n) S[(size_t)row * dm.m + m0 + l32] = acc[r] * dm.scale;
    }
  }
}

// Eight pooled queries per workgroup against the individual text keys, 256 tokens at a
// time (a multiple of the block size), then one log-sum-exp per (query, text block).
template <int D, int BLK>
__global__ __launch_bounds__(256) void text_mass_kernel(Dims dm, ScoreArgs a) {
  constexpr int NQ = 8;
  __shared__ float qs[NQ][D];
  __shared__ float u[NQ][256];
  const int bh = blockIdx.y;
  const int b = bh / dm.heads, h = bh % dm.heads;
  const int n0 = blockIdx.x * NQ;
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
      mx = wave_max(mx);
      float sum = 0.f;
      for (int i = lane; i < cnt; i += 64) sum += expf(u[r][j * BLK + i] - mx);
      sum = wave_sum(sum);
      if (lane == 0) L[(size_t)(n0 + r) * dm.m + dm.n + (int)(first / BLK)] = mx + logf(sum);
    }
    __syncthreads();
  }
}

// One wave per row, the row held in registers (rows of at most 64 * NI blocks), so every value
// is read once, every exponential is taken once and no barrier is needed.
template <int NI>
__global__ __launch_bounds__(256) void ipar_softmax_rows_kernel(Dims dm, ScoreArgs a) {
  const int wave = threadIdx.x / 64, lane = threadIdx.x % 64;
  const int n = blockIdx.x * 4 + wave, bh = blockIdx.y;
  if (n >= dm.n) return;                         // no barriers in this kernel
  const size_t row = ((size_t)bh * dm.n + n) * dm.m;
  const float* S = a.Spool + row;
  float* L = a.Lmass + row;
  float* A = a.Apool + row;
  const float ln_full = logf((float)dm.blk), ln_last = logf((float)dm.block_count(dm.n - 1));
  float l[NI];
  float mx = -INFINITY;
#pragma unroll
  for (int i = 0; i < NI; ++i) {
    const int m = lane + 64 * i;
    l[i] = -INFINITY;
    if (m < dm.m) {
      if (m < dm.n) {
        l[i] = S[m] + (m == dm.n - 1 ? ln_last : ln_full);
        L[m] = l[i];
      } else {
        l[i] = L[m];
      }
    }
    mx = fmaxf(mx, l[i]);
  }
  mx = wave_max(mx);
  float sum = 0.f;
#pragma unroll
  for (int i = 0; i < NI; ++i) {
    l[i] = expf(l[i] - mx);                      // exp(-inf) = 0 for the slots past the row end
    sum += l[i];
  }
  sum = wave_sum(sum);
  const float inv = 1.0f / sum;
#pragma unroll
  for (int i = 0; i < NI; ++i) {
    const int m = lane + 64 * i;
    if (m < dm.m) A[m] = l[i] * inv;
  }
}

template <int D, int BLK>
hipError_t launch_scores_t(const Dims& dm, const ScoreArgs& a, hipStream_t s) {
  const int bh = dm.batch * dm.heads;
  hipLaunchKernelGGL((pooled_scores_kernel<D>), dim3((dm.m + 63) / 64, (dm.n + 63) / 64, bh), dim3(256), 0, s, dm, a);
  if (dm.tt > 0)
    hipLaunchKernelGGL((text_mass_kernel<D, BLK>), dim3((dm.n + 7) / 8, bh), dim3(256), 0, s, dm, a);
  const dim3 rgrid((dm.n + 3) / 4, bh);
  if (dm.m <= 64 * 4)
    hipLaunchKernelGGL(ipar_softmax_rows_kernel<4>, rgrid, dim3(256), 0, s, dm, a);
  else if (dm.m <= 64 * 16)
    hipLaunchKernelGGL(ipar_softmax_rows_kernel<16>, rgrid, dim3(256), 0, s, dm, a);
  else if (dm.m <= 64 * 32)
    hipLaunchKernelGGL(ipar_softmax_rows_kernel<32>, rgrid, dim3(256), 0, s, dm, a);
  else
    hipLaunchKernelGGL(ipar_softmax_rows_kernel<RSA_MAX_BLOCKS / 64>, rgrid, dim3(256), 0, s, dm, a);
  return hipGetLastError();
}

}  // namespace

hipError_t launch_scores(const Dims& dm, const ScoreArgs& a, hipStream_t s) {
  if (dm.d == 128 && dm.blk == 128) return launch_scores_t<128, 128>(dm, a, s);
  if (dm.d == 128 && dm.blk == 64) return launch_scores_t<128, 64>(dm, a, s);
  if (dm.d == 64 && dm.blk == 128) return launch_scores_t<64, 128>(dm, a, s);
  return launch_scores_t<64, 64>(dm, a, s);
}

}  // namespace rsa
