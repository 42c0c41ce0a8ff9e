// Implicit full attention from pooled query-key interactions (paper Sec. 3.2, Sec. 4.1;
// Alg. 1 steps 5-7). Everything stays fp32: the selection that follows compares these
// values and is checked against an fp64 reference inside a 1e-4 band.
//
//   pooled_scores_kernel   Spool[n][m] = scale * q^pool_n . k^pool_m       (N x M x d, tiny)
//   text_mass_kernel       Lmass[n][N+i] = log sum_{t in text block i} exp(scale * q^pool_n . k_t)
//   ipar_softmax_rows_kernel  Lmass[n][m<N] = Spool + ln c_m ; Apool = row-softmax(Lmass)
//   ipar_fused_kernel      the first and the third in one pass (rows of at most 1024 blocks)
//
// softmax(Lmass) is the paper's reallocation written in log space: the mixed softmax
// over [pooled video keys ; text tokens] gives weights proportional to exp(score); a video
// block is then multiplied by its token count (exp(s + ln c)), text tokens are summed per
// block (exp(logsumexp)), and everything is divided by the row total.
#include <type_traits>

#include "lds_dma.hpp"
#include "rsa_common.hpp"
#include "text_mass.hpp"

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

// The text log-masses by themselves (text_mass.hpp has the work).
template <int D, int BLK>
__global__ __launch_bounds__(256) void text_mass_kernel(Dims dm, ScoreArgs a) {
  __shared__ float lds[text_mass_lds_floats<D>()];
  text_mass_block<D, BLK>(dm, a, blockIdx.x * kTextMassQueries, blockIdx.y, lds);
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

// Reduction over the 32 lanes of each half-wave with data-parallel-primitive moves (row shifts inside
// the rows of 16 lanes, then a row broadcast): lanes 31 and 63 end up with the result of their half.
template <bool MAX>
__device__ __forceinline__ float half_wave_reduce(float v) {
  constexpr int kIdentity = MAX ? (int)0xff800000u : 0;       // -inf or 0 for lanes without a source
  auto step = [&](auto ctrl, auto row_mask) __attribute__((always_inline)) {
    const int o = __builtin_amdgcn_update_dpp(kIdentity, __builtin_bit_cast(int, v), decltype(ctrl)::value,
                                              decltype(row_mask)::value, 0xf, false);
    const float f = __builtin_bit_cast(float, o);
    v = MAX ? fmaxf(v, f) : v + f;
  };
  step(std::integral_constant<int, 0x111>{}, std::integral_constant<int, 0xf>{});   // row_shr:1
  step(std::integral_constant<int, 0x112>{}, std::integral_constant<int, 0xf>{});   // row_shr:2
  step(std::integral_constant<int, 0x114>{}, std::integral_constant<int, 0xf>{});   // row_shr:4
  step(std::integral_constant<int, 0x118>{}, std::integral_constant<int, 0xf>{});   // row_shr:8
  step(std::integral_constant<int, 0x142>{}, std::integral_constant<int, 0xa>{});   // row_bcast:15 into rows 1 and 3
  return v;
}

// Alg. 1 steps 5-7 in one pass over the N x M tensors (rows of at most 128 * NT blocks): a workgroup
// owns 32 pooled queries and all M key blocks. Wave w takes the key tiles NT w .. NT w + NT - 1 (32
// blocks each: a band of consecutive columns). The product is v_mfma_f32_32x32x2_f32 as in
// pooled_scores_kernel, and every score of the wave's band stays in registers. Scores are written once
// (Spool), turned into log-masses (video blocks: + ln c_m; text blocks: what text_mass_kernel left in
// Lmass), and the row softmax is taken across the registers, the half-waves and the four waves, so
// that Lmass and Apool are written once too and nothing is read back. The text columns of Lmass must
// be in place before this kernel runs.
//
// Each wave has 16 KB of LDS to itself (two workgroups fit a CU, so that the epilogue of one runs
// beside the matrix work of the other):
//  - in the product, two buffers of half a key tile: the pooled keys come in with direct-to-LDS loads,
//    the contraction index in two halves (each half-wave's D/4 channels of the half), the half after the
//    one being multiplied always on its way. A buffer row is one key block: PPR 16-byte positions, the
//    lower half of them the channels of the lower half-wave; position p of row r holds logical chunk
//    p ^ (r mod PPR), so that lanes reading one logical chunk of different rows hit different banks;
//  - in the epilogue, a [32][32 * HT] tile of floats through which the accumulators (a lane holds one
//    column of 16 rows) are turned into rows, so that a store instruction writes two runs of 128 * HT
//    bytes instead of two of 128: a wave may have 63 stores in flight, and with narrow ones that bound,
//    not the memory, sets the pace.
typedef float floatx4_u __attribute__((ext_vector_type(4), aligned(4)));
template <int D, int NT>
__global__ __launch_bounds__(256, 2) void ipar_fused_kernel(Dims dm, ScoreArgs a) {
  constexpr int KH = D / 2;                     // k-steps; channels per half-wave
  constexpr int PPR = D / 8;                    // 16-byte positions per buffer row (half the channels of a key block)
  constexpr int HALF = 32 * PPR * 4;            // floats per buffer
  constexpr int RPL = 64 / PPR;                 // rows per load
  constexpr int LOADS = 32 / RPL;               // direct-to-LDS loads per half tile
  constexpr int HT = NT < 4 ? NT : 4;           // tiles per epilogue pass (HT * 4 KB <= the wave's LDS)
  static_assert(2 * HALF * 4 == 16384 || D == 64, "a wave's LDS: two half tiles");
  static_assert(32 * 32 * HT * 4 <= 2 * HALF * 4 || D == 64, "the epilogue tile fits the wave's LDS");
  constexpr int WAVE_LDS = (2 * HALF > 32 * 32 * HT) ? 2 * HALF : 32 * 32 * HT;   // floats
  __shared__ __attribute__((aligned(1024))) float wlds[4][WAVE_LDS];
  __shared__ float red[2][4][32];               // row maxima, then row sums, of each wave
  // Workgroups go round the 8 XCDs by their index; XCD x takes the (batch, head) pairs x, x + 8, ... one
  // after the other, so that the pooled keys its L2 serves at any time are those of a head or two.
  const int row_tiles = (dm.n + 31) / 32;
  const int xcd = blockIdx.x % 8, k = blockIdx.x / 8;
  const int bh = xcd + 8 * (k / row_tiles);
  if (bh >= dm.batch * dm.heads) return;        // the whole workgroup, before any barrier
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / 64), lane = threadIdx.x % 64;
  const int l32 = lane % 32, hf = lane / 32;
  const int n0 = (k % row_tiles) * 32;
  const int M = dm.m, N = dm.n;
  float* mine = wlds[wave];

  // this lane's pooled query (row n0 + l32, clamped: rows past the end are computed and not stored)
  floatx4 qv[KH / 4];
  {
    const int n = n0 + l32 < N ? n0 + l32 : N - 1;
    const floatx4* qrow = reinterpret_cast<const floatx4*>(a.Qp + ((size_t)bh * N + n) * D + hf * KH);
#pragma unroll
    for (int i = 0; i < KH / 4; ++i) qv[i] = qrow[i];
  }
  // the query must be in before the first direct-to-LDS load goes out: the compiler does not see those
  // loads and would wait for them together with the query at its first use
  __builtin_amdgcn_s_waitcnt(0x0F70);           // vmcnt(0)
  floatx16 acc[NT];
#pragma unroll
  for (int t = 0; t < NT; ++t)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[t][r] = 0.f;

  const int n_tiles = (M + 31) / 32;
  const float* Kp = a.Kp + (size_t)bh * M * D;
  const int lrow = lane / PPR, lpos = lane % PPR;
  // half c of key tile ct into buffer `buf`
  auto request_half = [&](int ct, int c, int buf) __attribute__((always_inline)) {
    const int m0 = ct * 32;
    const uint32_t dst = (uint32_t)(uintptr_t)(mine + buf * HALF);
#pragma unroll
    for (int j = 0; j < LOADS; ++j) {
      const int r = j * RPL + lrow;
      const int m = m0 + r < M ? m0 + r : M - 1;     // rows past the end repeat the last one (not stored)
      const int q = lpos ^ (r % PPR);                // logical chunk: half-wave q / (PPR/2), chunk q % (PPR/2) of this half
      const int ch = (q / (PPR / 2)) * KH + c * (KH / 2) + 4 * (q % (PPR / 2));
      dma16_v(dst + j * 1024, Kp + (size_t)m * D + ch, &wlds[0][0]);
    }
  };
  const int ct0 = wave * NT;
  if (ct0 < n_tiles) request_half(ct0, 0, 0);
#pragma unroll
  for (int t = 0; t < NT; ++t) {
    const int ct = ct0 + t;
    if (ct < n_tiles) {                          // wave-uniform
#pragma unroll
      for (int c = 0; c < 2; ++c) {
        // the buffer of the next half was last read two halves ago: those reads fed MFMAs that have been issued
        const bool more = c == 0 || (t + 1 < NT && ct + 1 < n_tiles);
        if (more) {
          request_half(c == 0 ? ct : ct + 1, 1 - c, 1 - c);
          wait_loads_leaving<LOADS>();
        } else {
          wait_loads_leaving<0>();
        }
        asm volatile("" ::: "memory");           // no read of the buffer may move above the wait
        const floatx4* kb = reinterpret_cast<const floatx4*>(mine + c * HALF) + l32 * PPR;
#pragma unroll
        for (int i = 0; i < KH / 8; ++i) {
          const floatx4 kq = kb[(hf * (PPR / 2) + i) ^ (l32 % PPR)];
#pragma unroll
          for (int e = 0; e < 4; ++e)
            acc[t] = __builtin_amdgcn_mfma_f32_32x32x2f32(qv[c * (KH / 8) + i][e], kq[e], acc[t], 0, 0, 0);
        }
      }
    }
  }

  // accumulator register r of tile t: query row n0 + 8(r/4) + 4*hf + r%4, key block 32*(NT*wave + t) + l32.
  const size_t row0 = (size_t)bh * N * M;
  float* S = a.Spool + row0;
  float* L = a.Lmass + row0;
  float* A = a.Apool + row0;
  const float ln_full = logf((float)dm.blk), ln_last = logf((float)dm.block_count(N - 1));
  const int band0 = ct0 * 32;                    // first column of the wave's band
  const int mcol = band0 + l32;                  // this lane's column in tile 0 of the band
  // Writes f(t, r) for every accumulator to rows n0 .. n0+31 of `out`, columns [band0, band0 + 32 NT) cut at
  // `col_end`, through the wave's LDS tile: HT tiles at a time, whole rows of the tile per store.
  auto store_band = [&](float* out, int col_end, auto f) __attribute__((always_inline)) {
    constexpr int TW = 32 * HT;                  // floats per tile row
#pragma unroll
    for (int p0 = 0; p0 < NT; p0 += HT) {
      asm volatile("" ::: "memory");
#pragma unroll
      for (int tt = 0; tt < HT; ++tt)
#pragma unroll
        for (int r = 0; r < 16; ++r) mine[(8 * (r / 4) + 4 * hf + (r % 4)) * TW + 32 * tt + l32] = f(p0 + tt, r);
      asm volatile("" ::: "memory");
      // a tile row is TW / 4 lanes of four floats: 64 lanes take RPI rows per store instruction.
      // The loop stays rolled: unrolled, all its addresses would be worked out ahead and spill.
      constexpr int LPR = TW / 4, RPI = 64 / LPR;
      const int rsub = lane / LPR, cl = 4 * (lane % LPR);
      const float* src = &mine[rsub * TW + cl];
      const int m = band0 + 32 * p0 + cl;
      float* dst = out + (size_t)(n0 + rsub) * M + m;
#pragma clang loop unroll(disable)
      for (int i = 0; i < 32 / RPI; ++i) {
        const int n = n0 + RPI * i + rsub;
        const floatx4 v = *reinterpret_cast<const floatx4*>(src);
        if (n < N) {
          if (m + 3 < col_end) {
            *reinterpret_cast<floatx4_u*>(dst) = v;
          } else {
#pragma unroll
            for (int e = 0; e < 3; ++e)
              if (m + e < col_end) dst[e] = v[e];
          }
        }
        src += RPI * TW;
        dst += RPI * (size_t)M;
      }
    }
  };
  // (the scores first, with nothing but stores in flight: a load in between would be waited for together
  // with every store before it)
  store_band(S, M, [&](int t, int r) __attribute__((always_inline)) { return acc[t][r] * dm.scale; });
  float pm[16];
#pragma unroll
  for (int r = 0; r < 16; ++r) pm[r] = -INFINITY;
#pragma unroll
  for (int t = 0; t < NT; ++t) {
    const int m = mcol + 32 * t;
    const int tile_first = (ct0 + t) * 32;
    if (tile_first + 32 <= N) {                  // wave-uniform: video blocks only, none of them the last
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        acc[t][r] = acc[t][r] * dm.scale + ln_full;
        pm[r] = fmaxf(pm[r], acc[t][r]);
      }
    } else {
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int n = n0 + 8 * (r / 4) + 4 * hf + (r % 4);
        float l = -INFINITY;
        if (m < N) l = acc[t][r] * dm.scale + (m == N - 1 ? ln_last : ln_full);
        else if (m < M) l = L[(size_t)(n < N ? n : N - 1) * M + m];
        acc[t][r] = l;
        pm[r] = fmaxf(pm[r], l);
      }
    }
  }
  // the log-masses of the video blocks (the text columns already hold theirs)
  store_band(L, N, [&](int t, int r) __attribute__((always_inline)) { return acc[t][r]; });
  // row maxima: over the lanes of the half-wave, then over the waves through LDS
#pragma unroll
  for (int r = 0; r < 16; ++r) {
    const float v = half_wave_reduce<true>(pm[r]);
    if (l32 == 31) red[0][wave][8 * (r / 4) + 4 * hf + (r % 4)] = v;
  }
  __syncthreads();
  float mx[16];
#pragma unroll
  for (int g = 0; g < 4; ++g) {
    floatx4 v = *reinterpret_cast<const floatx4*>(&red[0][0][8 * g + 4 * hf]);
#pragma unroll
    for (int w = 1; w < 4; ++w) {
      const floatx4 u = *reinterpret_cast<const floatx4*>(&red[0][w][8 * g + 4 * hf]);
#pragma unroll
      for (int e = 0; e < 4; ++e) v[e] = fmaxf(v[e], u[e]);
    }
#pragma unroll
    for (int e = 0; e < 4; ++e) mx[4 * g + e] = v[e];
  }
  float ps[16];
#pragma unroll
  for (int r = 0; r < 16; ++r) ps[r] = 0.f;
#pragma unroll
  for (int t = 0; t < NT; ++t)
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const float e = expf(acc[t][r] - mx[r]);    // exp(-inf) = 0 for the slots past the row end
      acc[t][r] = e;
      ps[r] += e;
    }
#pragma unroll
  for (int r = 0; r < 16; ++r) {
    const float v = half_wave_reduce<false>(ps[r]);
    if (l32 == 31) red[1][wave][8 * (r / 4) + 4 * hf + (r % 4)] = v;
  }
  __syncthreads();
  float inv[16];
#pragma unroll
  for (int g = 0; g < 4; ++g) {
    floatx4 v = *reinterpret_cast<const floatx4*>(&red[1][0][8 * g + 4 * hf]);
#pragma unroll
    for (int w = 1; w < 4; ++w) {
      const floatx4 u = *reinterpret_cast<const floatx4*>(&red[1][w][8 * g + 4 * hf]);
#pragma unroll
      for (int e = 0; e < 4; ++e) v[e] += u[e];
    }
#pragma unroll
    for (int e = 0; e < 4; ++e) inv[4 * g + e] = 1.0f / v[e];
  }
  store_band(A, M, [&](int t, int r) __attribute__((always_inline)) { return acc[t][r] * inv[r]; });
}

template <int D, int BLK>
hipError_t launch_scores_t(const Dims& dm, const ScoreArgs& a, hipStream_t s) {
  const int bh = dm.batch * dm.heads;
  if (dm.m <= 1024) {
    // rows short enough for the registers of a workgroup: the text log-masses first, then one pass
    if (dm.tt > 0 && !a.text_done)
      hipLaunchKernelGGL((text_mass_kernel<D, BLK>), dim3((dm.n + 7) / 8, bh), dim3(256), 0, s, dm, a);
    const dim3 fgrid(8 * ((bh + 7) / 8) * ((dm.n + 31) / 32));
    if (dm.m <= 256)
      hipLaunchKernelGGL((ipar_fused_kernel<D, 2>), fgrid, dim3(256), 0, s, dm, a);
    else if (dm.m <= 512)
      hipLaunchKernelGGL((ipar_fused_kernel<D, 4>), fgrid, dim3(256), 0, s, dm, a);
    else
      hipLaunchKernelGGL((ipar_fused_kernel<D, 8>), fgrid, dim3(256), 0, s, dm, a);
    return hipGetLastError();
  }
  hipLaunchKernelGGL((pooled_scores_kernel<D>), dim3((dm.m + 63) / 64, (dm.n + 63) / 64, bh), dim3(256), 0, s, dm, a);
  if (dm.tt > 0 && !a.text_done)
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
