// Block-sparse flash attention with the rectification fused into the epilogue
// (paper Sec. 3.1 sparse attention, Alg. 1 steps 16-17; Sec. 4.1 / 4.2, Alg. 1 steps 19-23).
//
// One workgroup per (batch*head, query block), one wave per 32 query rows. Video query
// blocks walk their compact, ascending list of critical key blocks; text query blocks
// (and every block under RSA_DENSE) walk all M key blocks. Key blocks are consumed in steps
// of 64 keys. For each step the K rows [64][d] and the channel-major V rows [d][64] are
// brought into LDS by direct-to-LDS loads (global_load_lds_dwordx4: no staging registers),
// double-buffered, issued one whole step ahead; one barrier per step hands the buffers
// over. Each wave then computes, with v_mfma_f32_32x32x16_bf16,
//     S^T = K Q^T      (M = key, N = query, k = channel)      -> accumulators: one query
//     O^T += V^T P^T   (M = channel, N = query, k = key)         column per lane
// so the online softmax is lane-local except for one exchange between the two half-waves,
// and the probabilities a lane holds after the first product are exactly the B operand it
// needs for the second (rsa_pool stores V in that key order).
// Epilogue: O = R_n * acc / l + C_n with C_n = sum_{m: not kept and M_c} A^pool[n][m] v^pool_m.
//
// MFMA-bound by design: 4*B*B*d flop per (query block, key block) pair against 2*B*d*2
// bytes of K/V traffic that is meant to come from L2 / Infinity Cache: workgroups that run
// at the same time work on neighbouring query blocks of the same head, and each XCD
// (workgroup id modulo 8) owns a contiguous range of query blocks. Two workgroups share a
// CU (64 KB of LDS and at most 256 VGPRs each) so one's softmax overlaps the other's MFMAs.
#include "rsa_common.hpp"

namespace rsa {
namespace {

constexpr float kLog2e = 1.4426950408889634f;
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
constexpr int KVS = 64;   // keys per step

template <int D, int BLK>
struct AttnCfg {
  static constexpr int QW = 32;             // query rows per wave
  static constexpr int NW = BLK / QW;       // waves per workgroup
  static constexpr int NTHR = 64 * NW;
  static constexpr int SPB = BLK / KVS;     // steps per key block
  static constexpr int KT = KVS / 32;       // key tiles of S^T per step
  static constexpr int KS = D / 16;         // k-steps of K Q^T
  static constexpr int DT = D / 32;         // channel tiles of O^T
  static constexpr int PC = KVS / 16;       // 16-key chunks per step
  static constexpr int KCPR = D / 8;        // 16-byte chunks per K row
  static constexpr int VCPR = KVS / 8;      // 16-byte chunks per V^T row of one step
  static constexpr int KINST = KVS * KCPR / 64;   // 1 KB direct-to-LDS loads per K step tile
  static constexpr int VINST = D * VCPR / 64;     // ... per V^T step tile
  static constexpr int KPW = KINST / NW;    // per wave
  static constexpr int VPW = VINST / NW;
  static_assert(KINST % NW == 0 && VINST % NW == 0, "loads must split evenly over the waves");
};

// LDS tiles are unpadded; the 16-byte chunk c of row r is stored at chunk position
// c ^ key(r) so that 16 consecutive rows read at one logical chunk index hit 16 different
// positions (all banks once). CPR = chunks per row (8 or 16).
template <int CPR>
__device__ __forceinline__ int swz_key(int r) { return (r / (16 / CPR)) & (CPR - 1); }
template <int CPR>
__device__ __forceinline__ int swizzled(int r, int c) { return r * CPR + (c ^ swz_key<CPR>(r)); }

// Exchange between the two half-waves (lane l <-> lane l^32) with v_permlane32_swap.
// The vector elements are copied to scalars before the bit casts: a bit cast applied
// directly to an element expression reads element 0 whatever the index.
__device__ __forceinline__ void half_wave_pair(float v, float& lo, float& hi) {
  const uint32_t u = __builtin_bit_cast(uint32_t, v);
  const auto r = __builtin_amdgcn_permlane32_swap(u, u, false, false);
  const uint32_t r0 = r[0], r1 = r[1];
  lo = __builtin_bit_cast(float, r0);   // value held by lane l%32
  hi = __builtin_bit_cast(float, r1);   // value held by lane l%32 + 32
}
__device__ __forceinline__ float half_wave_max(float v) {
  float lo, hi;
  half_wave_pair(v, lo, hi);
  return fmaxf(lo, hi);
}
__device__ __forceinline__ float half_wave_sum(float v) {
  float lo, hi;
  half_wave_pair(v, lo, hi);
  return lo + hi;
}

// Direct-to-LDS loads (global_load_lds_dwordx4): every lane supplies the address of 16
// bytes; lane L's data lands at lds_addr + 16*L, lds_addr wave-uniform (goes to M0). The
// compiler does not track these loads: the caller waits with s_waitcnt vmcnt before the
// barrier that publishes the buffer, and `fence` names the LDS buffer so that it counts as
// written. Two address forms: scalar base + per-lane 32-bit byte offset, and per-lane pointer.
__device__ __forceinline__ void dma16_sv(uint32_t lds_addr, const void* sbase, uint32_t voff, void* fence) {
  asm volatile("s_mov_b32 m0, %0\n\tglobal_load_lds_dwordx4 %1, %2"
               ::"s"(lds_addr), "v"(voff), "s"(sbase), "r"(fence) : "memory");
}
__device__ __forceinline__ void dma16_v(uint32_t lds_addr, const void* gptr, void* fence) {
  asm volatile("s_mov_b32 m0, %0\n\tglobal_load_lds_dwordx4 %1, off" ::"s"(lds_addr), "v"(gptr), "r"(fence) : "memory");
}
__device__ __forceinline__ void wait_all_loads() { __builtin_amdgcn_s_waitcnt(0x0F70); }   // vmcnt(0)

// The running softmax reference is only raised when a row's new maximum exceeds it by
// more than this many binades; probabilities then stay below 2^kLazyBits, which fp32 sums
// and bf16 operands hold without loss, and the accumulators are rescaled rarely.
constexpr float kLazyBits = 6.0f;

template <int V>
struct IntC { static constexpr int value = V; };

template <int D, int BLK>
__global__ __launch_bounds__(64 * BLK / 32, (BLK == 128 ? 2 : 1)) void attn_kernel(Dims dm, AttnArgs a, int n_text_items, int chunk) {
  using C = AttnCfg<D, BLK>;
  constexpr int KBUF = KVS * C::KCPR, VBUF = D * C::VCPR;    // 16-byte chunks per buffer
  __shared__ u32x4 ldsK[2 * KBUF];
  __shared__ u32x4 ldsV[2 * VBUF];
  __shared__ float comp[2][D];

  // ---- which (batch*head, query block) is this workgroup ---------------------------------
  const bool dense_all = (a.flags & RSA_DENSE) != 0;
  int bh, qb;
  {
    const int id = blockIdx.x;
    if (id < n_text_items) {           // long dense rows first
      const int per = dense_all ? dm.m : dm.mt;
      bh = id / per;
      qb = dense_all ? id % per : dm.n + id % per;
    } else {
      const int v = id - n_text_items;
      const int xcd = v & 7, j = v >> 3;
      bh = j / chunk;
      qb = xcd * chunk + j % chunk;
      if (qb >= dm.n) return;
    }
  }
  const int b = bh / dm.heads, h = bh % dm.heads;
  const bool sparse_row = !dense_all && qb < dm.n;
  const size_t vrow = (size_t)bh * dm.n + qb;      // row of the per-video-block tensors
  const int nlist = sparse_row ? a.count[vrow] : dm.m;
  const int32_t* list = sparse_row ? a.block_idx + vrow * dm.m : nullptr;

  const int tid = threadIdx.x;
  const int wave = __builtin_amdgcn_readfirstlane(tid / 64);   // wave-uniform: lives in an SGPR
  const int lane = tid % 64;
  const int l32 = lane % 32, hf = lane / 32;
  const int64_t base = (int64_t)b * dm.sb + (int64_t)h * dm.sh;
  const uint16_t* Qb = a.Q + base;
  const uint16_t* Kb = a.K + base;
  const uint16_t* Vtb = a.Vt + (size_t)bh * dm.m * D * BLK;

  // ---- pooled compensation C_n (Alg. 1 step 21), parked in LDS for the epilogue ----------
  const bool do_comp = sparse_row && (a.flags & RSA_COMPENSATE);
  if (do_comp) {
    constexpr int G = C::NTHR / D;                 // thread groups striding over mask words
    const int dd = tid % D, g = tid / D;
    float accv = 0.f;
    if (g < 2) {
      const uint32_t* mk = a.mask_bits + vrow * dm.w;
      const uint32_t* mc = a.Mc_bits + vrow * dm.w;
      const float* Ap = a.Apool + vrow * dm.m;
      const float* Vp = a.Vp + (size_t)bh * dm.m * D;
      constexpr int GS = G < 2 ? G : 2;
      for (int wd = g; wd < dm.w; wd += GS) {
        uint32_t bits = ~mk[wd] & mc[wd];
        while (bits) {
          const int bit = __builtin_ctz(bits);
          bits &= bits - 1;
          const int m = wd * 32 + bit;
          accv = fmaf(Ap[m], Vp[(size_t)m * D + dd], accv);
        }
      }
      comp[g][dd] = accv;
    }
    if (G < 2 && tid < D) comp[1][tid] = 0.f;
  }

  // ---- loop-invariant per-lane pieces of the direct-to-LDS loads --------------------------
  // Load i of a K step tile fills LDS rows [i*RK, (i+1)*RK); wave w issues loads w*KPW + ii.
  constexpr int RK = 64 / C::KCPR, RV = 64 / C::VCPR;
  int k_row[C::KPW], k_col[C::KPW];
  uint32_t k_voff[C::KPW], v_voff[C::VPW];       // byte offsets from the step's scalar base
#pragma unroll
  for (int ii = 0; ii < C::KPW; ++ii) {
    const int r = (wave * C::KPW + ii) * RK + lane / C::KCPR;
    k_row[ii] = r;
    k_col[ii] = ((lane % C::KCPR) ^ swz_key<C::KCPR>(r)) * 8;
    k_voff[ii] = (uint32_t)((r * dm.st + k_col[ii]) * 2);
  }
#pragma unroll
  for (int ii = 0; ii < C::VPW; ++ii) {
    const int dd = (wave * C::VPW + ii) * RV + lane / C::VCPR;
    v_voff[ii] = (uint32_t)((dd * BLK + ((lane % C::VCPR) ^ swz_key<C::VCPR>(dd)) * 8) * 2);
  }
  const uint32_t ldsK_addr = (uint32_t)(uintptr_t)&ldsK[0] + wave * C::KPW * 1024;
  const uint32_t ldsV_addr = (uint32_t)(uintptr_t)&ldsV[0] + wave * C::VPW * 1024;

  // Requests the K rows and V^T rows of step `half` of key block m into buffer `buf`.
  auto issue_step = [&](int m, int half, int buf) {
    const int kv_count = dm.block_count(m);
    const uint16_t* kblk = Kb + dm.block_start(m) * dm.st;
    const uint32_t kdst = ldsK_addr + buf * (KBUF * 16), vdst = ldsV_addr + buf * (VBUF * 16);
    if (kv_count == BLK) {
      const uint16_t* ksrc = kblk + (int64_t)(half * KVS) * dm.st;
#pragma unroll
      for (int ii = 0; ii < C::KPW; ++ii) dma16_sv(kdst + ii * 1024, ksrc, k_voff[ii], ldsK);
    } else {
#pragma unroll
      for (int ii = 0; ii < C::KPW; ++ii) {
        int r = half * KVS + k_row[ii];
        r = r < kv_count ? r : kv_count - 1;   // rows past a ragged block re-read its last row (masked later)
        dma16_v(kdst + ii * 1024, kblk + (int64_t)r * dm.st + k_col[ii], ldsK);
      }
    }
    const uint16_t* vsrc = Vtb + (size_t)m * D * BLK + half * KVS;
#pragma unroll
    for (int ii = 0; ii < C::VPW; ++ii) dma16_sv(vdst + ii * 1024, vsrc, v_voff[ii], ldsV);
  };

  // ---- loop-invariant LDS read positions (16-byte chunk index inside buffer 0, tile 0) ----
  const u32x4* kread[C::KS];
  const u32x4* vread[C::PC];
#pragma unroll
  for (int ks = 0; ks < C::KS; ++ks) kread[ks] = ldsK + swizzled<C::KCPR>(l32, 2 * ks + hf);
#pragma unroll
  for (int pc = 0; pc < C::PC; ++pc) vread[pc] = ldsV + swizzled<C::VCPR>(l32, 2 * pc + hf);

  // ---- Q as the B operand of S^T = K Q^T, resident in registers --------------------------
  const int q_count = dm.block_count(qb);
  const int64_t q_t0 = dm.block_start(qb);
  bf16x8 qreg[C::KS];
  {
    const int q = wave * 32 + l32;
#pragma unroll
    for (int s = 0; s < C::KS; ++s) {
      uint4 v = make_uint4(0, 0, 0, 0);
      if (q < q_count) v = *reinterpret_cast<const uint4*>(Qb + (q_t0 + q) * dm.st + 16 * s + 8 * hf);
      qreg[s] = __builtin_bit_cast(bf16x8, v);
    }
  }

  floatx16 oacc[C::DT];
#pragma unroll
  for (int dt = 0; dt < C::DT; ++dt)
#pragma unroll
    for (int r = 0; r < 16; ++r) oacc[dt][r] = 0.f;
  float mref = -INFINITY, lpart = 0.f;   // softmax reference (log2 domain) and this lane's partial row sum
  const float cs = dm.scale * kLog2e;

  // One step: 64 keys of block m_cur from buffer BUF (compile-time, so every LDS offset is
  // an immediate), after requesting the following step into the other buffer.
  auto step = [&](auto bufc, int half, int m_cur, bool more, int m_next, int half_next) {
    constexpr int BUF = decltype(bufc)::value;
    const int kv_count = dm.block_count(m_cur);
    wait_all_loads();      // this wave's share of the step has landed
    __syncthreads();       // ... and everyone's; every wave is past the previous step, so the other buffer is free
    if (more) issue_step(m_next, half_next, BUF ^ 1);

    // ---- S^T = K Q^T: all K operands of the step are requested from LDS up front ---------
    bf16x8 kop[C::KS][C::KT];
#pragma unroll
    for (int ks = 0; ks < C::KS; ++ks)
#pragma unroll
      for (int t = 0; t < C::KT; ++t)
        kop[ks][t] = __builtin_bit_cast(bf16x8, kread[ks][BUF * KBUF + t * 32 * C::KCPR]);
    __builtin_amdgcn_sched_barrier(0);
    floatx16 sacc[C::KT];
#pragma unroll
    for (int t = 0; t < C::KT; ++t)
#pragma unroll
      for (int r = 0; r < 16; ++r) sacc[t][r] = 0.f;
#pragma unroll
    for (int ks = 0; ks < C::KS; ++ks)
#pragma unroll
      for (int t = 0; t < C::KT; ++t)
        sacc[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kop[ks][t], qreg[ks], sacc[t], 0, 0, 0);
    __builtin_amdgcn_sched_barrier(0);

    // accumulator register r of key tile t is key half*64 + 32t + 8(r/4) + 4*hf + r%4 of the block
    if (kv_count < BLK) {
#pragma unroll
      for (int t = 0; t < C::KT; ++t)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int kv = half * KVS + 32 * t + 8 * (r / 4) + 4 * hf + (r % 4);
          if (kv >= kv_count) sacc[t][r] = -INFINITY;
        }
    }

    // ---- online softmax, one query column per lane -----------------------------------
    float mx = -INFINITY;
#pragma unroll
    for (int t = 0; t < C::KT; ++t)
#pragma unroll
      for (int r = 0; r < 16; ++r) mx = fmaxf(mx, sacc[t][r]);
    mx = half_wave_max(mx) * cs;
    if (__any(mx > mref + kLazyBits)) {
      const float mnew = fmaxf(mref, mx);
      const float alpha = __builtin_amdgcn_exp2f(mref - mnew);
      mref = mnew;
      lpart *= alpha;
#pragma unroll
      for (int dt = 0; dt < C::DT; ++dt)
#pragma unroll
        for (int r = 0; r < 16; ++r) oacc[dt][r] *= alpha;
    }
    const float moff = -mref;
    u32x4 pb[C::PC];   // probabilities as bf16 B operands, 16 keys per entry
    float rs = 0.f;
#pragma unroll
    for (int t = 0; t < C::KT; ++t) {
      float p[16];
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        p[r] = __builtin_amdgcn_exp2f(fmaf(sacc[t][r], cs, moff));
        rs += p[r];
      }
#pragma unroll
      for (int u = 0; u < 2; ++u) {
        u32x4 w;
        w.x = pack_bf16x2(p[8 * u + 0], p[8 * u + 1]);
        w.y = pack_bf16x2(p[8 * u + 2], p[8 * u + 3]);
        w.z = pack_bf16x2(p[8 * u + 4], p[8 * u + 5]);
        w.w = pack_bf16x2(p[8 * u + 6], p[8 * u + 7]);
        pb[2 * t + u] = w;
      }
    }
    lpart += rs;
    __builtin_amdgcn_sched_barrier(0);

    // ---- O^T += V^T P^T: all V operands requested up front ---------------------------------
    bf16x8 vop[C::PC][C::DT];
#pragma unroll
    for (int pc = 0; pc < C::PC; ++pc)
#pragma unroll
      for (int dt = 0; dt < C::DT; ++dt)
        vop[pc][dt] = __builtin_bit_cast(bf16x8, vread[pc][BUF * VBUF + dt * 32 * C::VCPR]);
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int pc = 0; pc < C::PC; ++pc)
#pragma unroll
      for (int dt = 0; dt < C::DT; ++dt)
        oacc[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vop[pc][dt], __builtin_bit_cast(bf16x8, pb[pc]), oacc[dt], 0, 0, 0);
  };

  // Steps alternate between the two buffers; with two steps per key block the buffer index
  // is the half index, with one step per block the blocks alternate.
  if (nlist > 0) {
    int m_cur = list ? list[0] : 0;
    issue_step(m_cur, 0, 0);
    if constexpr (C::SPB == 2) {
      for (int j = 0; j < nlist; ++j) {
        const bool more = j + 1 < nlist;
        const int m_next = more ? (list ? list[j + 1] : j + 1) : m_cur;
        step(IntC<0>{}, 0, m_cur, true, m_cur, 1);
        step(IntC<1>{}, 1, m_cur, more, m_next, 0);
        m_cur = m_next;
      }
    } else {
      for (int j = 0; j < nlist; j += 2) {
        const bool more1 = j + 1 < nlist, more2 = j + 2 < nlist;
        const int m1 = more1 ? (list ? list[j + 1] : j + 1) : m_cur;
        const int m2 = more2 ? (list ? list[j + 2] : j + 2) : m1;
        step(IntC<0>{}, 0, m_cur, more1, m1, 0);
        if (more1) step(IntC<1>{}, 0, m1, more2, m2, 0);
        m_cur = m2;
      }
    }
  }

  // ---- epilogue: normalise, rectify, compensate, store ------------------------------------
  __syncthreads();   // comp[] is complete
  const float rfac = (sparse_row && (a.flags & RSA_RECTIFY_CRITICAL)) ? a.R[vrow] : 1.0f;
  uint16_t* Ob = a.O + base;
  {
    const float lsum = half_wave_sum(lpart);
    const int q = wave * 32 + l32;
    if (q < q_count) {
      const float f = rfac / lsum;
      uint16_t* orow = Ob + (q_t0 + q) * dm.st;
#pragma unroll
      for (int dt = 0; dt < C::DT; ++dt)
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          const int d0 = 32 * dt + 8 * g + 4 * hf;
          float o[4];
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            o[e] = oacc[dt][4 * g + e] * f;
            if (do_comp) o[e] += comp[0][d0 + e] + comp[1][d0 + e];
          }
          uint2 w;
          w.x = pack_bf16x2(o[0], o[1]);
          w.y = pack_bf16x2(o[2], o[3]);
          *reinterpret_cast<uint2*>(orow + d0) = w;
        }
      if (a.lse && hf == 0)
        a.lse[((size_t)bh * dm.t) + q_t0 + q] = (mref + log2f(lsum)) * 0.6931471805599453f;
    }
  }
}

template <int D, int BLK>
hipError_t launch_attn_t(const Dims& dm, const AttnArgs& a, hipStream_t s) {
  using C = AttnCfg<D, BLK>;
  const int bh = dm.batch * dm.heads;
  const bool dense_all = (a.flags & RSA_DENSE) != 0;
  const int n_text_items = dense_all ? bh * dm.m : bh * dm.mt;
  const int chunk = (dm.n + 7) / 8;
  const long long grid = (long long)n_text_items + (dense_all ? 0 : (long long)bh * 8 * chunk);
  if (grid <= 0 || grid > 0x7fffffffLL) return hipErrorInvalidValue;
  hipLaunchKernelGGL((attn_kernel<D, BLK>), dim3((unsigned)grid), dim3(C::NTHR), 0, s, dm, a, n_text_items, chunk);
  return hipGetLastError();
}

}  // namespace

hipError_t launch_attn(const Dims& dm, const AttnArgs& a, hipStream_t s) {
  if (dm.d == 128 && dm.blk == 128) return launch_attn_t<128, 128>(dm, a, s);
  if (dm.d == 128 && dm.blk == 64) return launch_attn_t<128, 64>(dm, a, s);
  if (dm.d == 64 && dm.blk == 128) return launch_attn_t<64, 128>(dm, a, s);
  return launch_attn_t<64, 64>(dm, a, s);
}

}  // namespace rsa
