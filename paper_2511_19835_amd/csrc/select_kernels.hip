// Sparse-mask generation and rectification factor (paper Alg. 1 steps 13-14 and 19;
// Sec. 4.1 for R_n, Sec. 4.3 and the appendix "Implementations" for top-k and p).
//
// One wavefront per video query block. The row's M log-masses become order-preserving
// 32-bit keys in registers, lane l owning blocks l, l+64, ... (four rows per workgroup, the
// register count chosen by the row length); the k-th largest key is found
// by a 32-step bitwise search whose counts are wave ballots, so the selection is exact
// integer work (ties: lower block index first). The optional weight threshold p extends
// the kept prefix, in the same descending order, until the kept A^pool exceeds p.
// Outputs: mask bits, ascending block list, count, and R_n = sum of kept A^pool.
#include <type_traits>

#include "rsa_common.hpp"

namespace rsa {
namespace {

__device__ inline uint32_t orderable_key(float x) {
  const uint32_t u = __builtin_bit_cast(uint32_t, x);
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}
__device__ inline int lanes_below(unsigned long long mask) {
  return __builtin_amdgcn_mbcnt_hi((uint32_t)(mask >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)mask, 0));
}
// Sum over the 64 lanes with data-parallel-primitive moves (row shifts inside the rows of 16 lanes, then
// the two row broadcasts); every lane gets the total.
__device__ inline float wave_sum(float v) {
  auto step = [&](auto ctrl, auto row_mask) __attribute__((always_inline)) {
    const int o = __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), decltype(ctrl)::value,
                                              decltype(row_mask)::value, 0xf, false);
    v += __builtin_bit_cast(float, o);
  };
  step(std::integral_constant<int, 0x111>{}, std::integral_constant<int, 0xf>{});   // row_shr:1
  step(std::integral_constant<int, 0x112>{}, std::integral_constant<int, 0xf>{});   // row_shr:2
  step(std::integral_constant<int, 0x114>{}, std::integral_constant<int, 0xf>{});   // row_shr:4
  step(std::integral_constant<int, 0x118>{}, std::integral_constant<int, 0xf>{});   // row_shr:8
  step(std::integral_constant<int, 0x142>{}, std::integral_constant<int, 0xa>{});   // row_bcast:15 into rows 1 and 3
  step(std::integral_constant<int, 0x143>{}, std::integral_constant<int, 0xc>{});   // row_bcast:31 into rows 2 and 3
  return __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), 63));
}
__device__ inline uint32_t wave_max_u32(uint32_t v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = max(v, (uint32_t)__shfl_xor((int)v, o));
  return v;
}
__device__ inline float wave_inclusive_scan(float v, int lane) {
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) {
    const float up = __shfl_up(v, o);
    if (lane >= o) v += up;
  }
  return v;
}

// Keys and weights of a row in NI registers per lane (rows of up to 64 * NI blocks), one row per
// wave of the workgroup.
template <int NI>
__global__ __launch_bounds__(256) void select_kernel(Dims dm, SelectArgs a) {
  const int lane = threadIdx.x % 64;
  const int n = blockIdx.x * 4 + (int)(threadIdx.x / 64), bh = blockIdx.y;
  if (n >= dm.n) return;                           // no barriers in this kernel
  const int M = dm.m;
  constexpr int slots = NI;
  const size_t row = (size_t)bh * dm.n + n;
  const float* L = a.Lmass + row * M;
  const float* A = a.Apool + row * M;
  uint32_t rk[NI];
  float rv[NI];
  auto key_at = [&](int s) __attribute__((always_inline)) { return rk[s]; };
  auto val_at = [&](int s) __attribute__((always_inline)) { return rv[s]; };

#pragma unroll
  for (int s = 0; s < slots; ++s) {
    const int m = s * 64 + lane;
    rk[s] = (m < M) ? orderable_key(L[m]) : 0u;   // 0 sorts below every real key
    rv[s] = (m < M) ? A[m] : 0.f;
  }

  // k-th largest key. The bits that all keys of the row share need no search (a candidate with such a
  // bit set is below or at every key, one with it clear above every key), and the search ends as soon as
  // a candidate is matched or passed by exactly `keep` keys: those are the kept blocks, whatever the
  // lower bits of the k-th key.
  uint32_t kmax = 0, nkmin = 0;
#pragma unroll
  for (int s = 0; s < slots; ++s) {
    const bool valid = s * 64 + lane < M;
    kmax = max(kmax, key_at(s));
    nkmin = max(nkmin, valid ? ~key_at(s) : 0u);
  }
  kmax = wave_max_u32(kmax);
  const uint32_t kmin = ~wave_max_u32(nkmin);
  const int vary = 32 - __builtin_clz((kmax ^ kmin) | 1u);      // low bits in which keys of this row differ (at least 1)
  uint32_t tau = vary >= 32 ? 0u : (kmax >> vary) << vary;
  bool exact = false;
  for (int bit = vary - 1; bit >= 0 && !exact; --bit) {
    const uint32_t cand = tau | (1u << bit);
    int cnt = 0;
    _Pragma("unroll") for (int s = 0; s < slots; ++s) cnt += __popcll(__ballot(key_at(s) >= cand));
    if (cnt >= a.keep) tau = cand;
    if (cnt == a.keep) {
      tau = cand - 1;             // "key > tau" is "key >= cand"; no key equal to tau is kept
      exact = true;
    }
  }
  int n_gt = 0;
  _Pragma("unroll") for (int s = 0; s < slots; ++s) n_gt += __popcll(__ballot(key_at(s) > tau));
  int ties = a.keep - n_gt;       // how many blocks equal to tau are kept (index order)
  int kept_target = a.keep;

  if (a.p > 0.f) {
    // largest threshold whose kept weight exceeds p
    uint32_t tau_p = 0;
    for (int bit = 31; bit >= 0; --bit) {
      const uint32_t cand = tau_p | (1u << bit);
      float part = 0.f;
      _Pragma("unroll") for (int s = 0; s < slots; ++s) part += (key_at(s) >= cand) ? val_at(s) : 0.f;
      if (wave_sum(part) > a.p) tau_p = cand;
    }
    float part = 0.f;
    int n_gt_p = 0;
#pragma unroll
    for (int s = 0; s < slots; ++s) {
      const bool gt = key_at(s) > tau_p;
      part += gt ? val_at(s) : 0.f;
      n_gt_p += __popcll(__ballot(gt));
    }
    float run = wave_sum(part);    // weight strictly above tau_p: not yet above p
    int ties_p = 0;
    if (tau_p != 0) {
#pragma unroll
      for (int s = 0; s < slots; ++s) {
        const bool tie = key_at(s) == tau_p;
        const float tv = tie ? val_at(s) : 0.f;
        const float incl = wave_inclusive_scan(tv, lane);
        ties_p += __popcll(__ballot(tie && (run + (incl - tv) <= a.p)));
        run += __shfl(incl, 63);
      }
    }
    if (n_gt_p + ties_p > kept_target) {
      kept_target = n_gt_p + ties_p;
      tau = tau_p;
      ties = ties_p;
    }
  }

  const uint32_t* forced = a.forced ? a.forced + row * dm.w : nullptr;
  uint32_t* mbits = a.mask_bits + row * dm.w;
  int32_t* list = a.block_idx + row * M;
  int list_base = 0, tie_base = 0;
  float rpart = 0.f;
#pragma unroll
  for (int s = 0; s < slots; ++s) {
    const int m = s * 64 + lane;
    const uint32_t key = key_at(s);
    const bool tie = key == tau && m < M;
    const unsigned long long tie_mask = __ballot(tie);
    bool kept = (key > tau) || (tie && (tie_base + lanes_below(tie_mask) < ties));
    tie_base += __popcll(tie_mask);
    const int word = 2 * s + (lane >> 5);
    if (forced && m < M) kept = kept || ((forced[word] >> (lane & 31)) & 1u);
    const unsigned long long kept_mask = __ballot(kept);
    if ((lane & 31) == 0 && word < dm.w) mbits[word] = (uint32_t)(kept_mask >> (lane & 32));
    if (kept) {
      list[list_base + lanes_below(kept_mask)] = m;
      rpart += val_at(s);
    }
    list_base += __popcll(kept_mask);
  }
  const float r = wave_sum(rpart);
  if (lane == 0) {
    a.count[row] = list_base;
    a.R[row] = r;
  }
}

}  // namespace

hipError_t launch_select(const Dims& dm, const SelectArgs& a, hipStream_t s) {
  const dim3 grid((dm.n + 3) / 4, dm.batch * dm.heads), block(256);
  if (dm.m <= 64 * 4)
    hipLaunchKernelGGL(select_kernel<4>, grid, block, 0, s, dm, a);
  else if (dm.m <= 64 * 16)
    hipLaunchKernelGGL(select_kernel<16>, grid, block, 0, s, dm, a);
  else if (dm.m <= 64 * 32)
    hipLaunchKernelGGL(select_kernel<32>, grid, block, 0, s, dm, a);
  else
    hipLaunchKernelGGL(select_kernel<RSA_MAX_BLOCKS / 64>, grid, block, 0, s, dm, a);
  return hipGetLastError();
}

}  // namespace rsa
