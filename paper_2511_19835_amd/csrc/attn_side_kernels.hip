// The small kernels that run before the persistent attention kernel (paper Alg. 1 step 21 for the pooled
// compensation; the launch order and the schedule are this library's own): compensation_kernel,
// row_order_kernel, schedule_kernel, and compensation_schedule_kernel = the first and the third in one launch.
#include "attn_sched.hpp"

namespace rsa {
namespace {

// Pooled compensation (Alg. 1 step 21): C[n][:] = sum over blocks m that are not kept and
// have their M_c bit set of A^pool[n][m] * v^pool[m][:], all fp32. Written as the product it is:
// W V^pool with W[n][m] = A^pool[n][m] where block m is compensated for row n and 0 elsewhere
// (about a fifth of the entries at the benchmark shape), on v_mfma_f32_32x32x2_f32 -- fp32 operands,
// fp32 products and sums. One workgroup per 32 query blocks of a (batch, head); the key blocks come
// 64 at a time: the weights of the 32 rows (read whole, masked on their way into LDS) and the 64 rows
// of v^pool go through LDS, the next 64 are on their way while
// the matrix instructions of these run; wave w owns channels 32 w .. 32 w + 31 (M = query row,
// N = channel, k = key block: the lower half-wave takes blocks 8u .. 8u+3 of a run of eight, the
// upper one 8u+4 .. 8u+7, both operands alike). Blocks past the end of the row carry weight 0.
// v^pool of a head is read once per workgroup (from L2) instead of once per compensated pair.
constexpr int kCompChunk = 64;                   // key blocks per pass
constexpr int kCompStride = kCompChunk + 4;      // floats per row of the weight tile (16-byte rows, spread over the banks)
template <int D>
constexpr unsigned comp_lds_bytes() { return (32 * kCompStride + kCompChunk * D) * 4; }

template <int D>
__device__ __forceinline__ void compensate_tile(const Dims& dm, const AttnArgs& a, int n0, int bh, uint32_t* lds) {
  constexpr int MC = kCompChunk, AS = kCompStride;
  constexpr int CT = D / 32;                     // channel tiles = waves with matrix work
  constexpr int VL = MC * D / 4 / 256;           // 16-byte loads of v^pool per thread and pass
  float* wt = reinterpret_cast<float*>(lds);     // [32][AS]
  float* vt = wt + 32 * AS;                      // [MC][D]
  const int tid = threadIdx.x;
  const int wave = __builtin_amdgcn_readfirstlane(tid / 64), lane = tid % 64, l32 = lane % 32, hf = lane / 32;
  const float* Vp = a.Vp + (size_t)bh * dm.m * D;
  // this thread's share of the weight tile: row tid / 8, the eight blocks from 8 (tid % 8) on (one mask word)
  const int wr = tid / 8, wc = (tid % 8) * 8;
  const bool row_ok = n0 + wr < dm.n;
  const size_t row = (size_t)bh * dm.n + (row_ok ? n0 + wr : dm.n - 1);
  const uint32_t* kept = a.mask_bits + row * dm.w;
  const uint32_t* gate = a.Mc_bits + row * dm.w;
  const float* A = a.Apool + row * dm.m;
  float w[8];
  uint32_t on = 0u;                              // bits of this thread's eight blocks: compensated or not
  floatx4 vv[VL];
  typedef float floatx4_u __attribute__((ext_vector_type(4), aligned(4)));     // rows of A^pool start at any word
  // Nothing here depends on anything else loaded here: the weights are read whole and masked when they go to LDS.
  auto fetch = [&](int m0) __attribute__((always_inline)) {
    const int m = m0 + wc;
    on = 0u;
#pragma unroll
    for (int e = 0; e < 8; ++e) w[e] = 0.f;
    if (row_ok && m < dm.m) {
      on = (~kept[m / 32] & gate[m / 32]) >> (m % 32);
      if (m + 8 <= dm.m) {
        const floatx4 lo = *reinterpret_cast<const floatx4_u*>(A + m), hi = *reinterpret_cast<const floatx4_u*>(A + m + 4);
#pragma unroll
        for (int e = 0; e < 4; ++e) { w[e] = lo[e]; w[4 + e] = hi[e]; }
      } else {
#pragma unroll
        for (int e = 0; e < 8; ++e) if (m + e < dm.m) w[e] = A[m + e];
      }
    }
#pragma unroll
    for (int i = 0; i < VL; ++i) {
      const int idx = tid + 256 * i, r = idx / (D / 4), c4 = idx % (D / 4);
      const int mm = m0 + r < dm.m ? m0 + r : dm.m - 1;        // rows past the end repeat the last one (weight 0)
      vv[i] = *reinterpret_cast<const floatx4*>(Vp + (size_t)mm * D + 4 * c4);
    }
  };
  floatx16 acc;
#pragma unroll
  for (int r = 0; r < 16; ++r) acc[r] = 0.f;
  fetch(0);
  for (int m0 = 0; m0 < dm.m; m0 += MC) {
    __syncthreads();                             // the tiles of the pass before have been read
#pragma unroll
    for (int e = 0; e < 8; ++e) w[e] = ((on >> e) & 1u) ? w[e] : 0.f;
    *reinterpret_cast<floatx4*>(wt + wr * AS + wc) = floatx4{w[0], w[1], w[2], w[3]};
    *reinterpret_cast<floatx4*>(wt + wr * AS + wc + 4) = floatx4{w[4], w[5], w[6], w[7]};
#pragma unroll
    for (int i = 0; i < VL; ++i) {
      const int idx = tid + 256 * i;
      *reinterpret_cast<floatx4*>(vt + 4 * idx) = vv[i];      // row idx / (D/4), chunk idx % (D/4): rows are D floats
    }
    __syncthreads();
    if (m0 + MC < dm.m) fetch(m0 + MC);
    if (wave < CT) {
#pragma unroll
      for (int u = 0; u < MC / 8; ++u) {
        const floatx4 a4 = *reinterpret_cast<const floatx4*>(wt + l32 * AS + 8 * u + 4 * hf);
#pragma unroll
        for (int e = 0; e < 4; ++e)
          acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a4[e], vt[(8 * u + 4 * hf + e) * D + 32 * wave + l32], acc, 0, 0, 0);
      }
    }
  }
  // accumulator register r: query block n0 + 8(r/4) + 4*hf + r%4, channel 32*wave + l32
  if (wave < CT) {
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const int n = n0 + 8 * (r / 4) + 4 * hf + (r % 4);
      if (n < dm.n) a.comp[((size_t)bh * dm.n + n) * D + 32 * wave + l32] = acc[r];
    }
  }
}

template <int D>
__global__ __launch_bounds__(256) void compensation_kernel(Dims dm, AttnArgs a) {
  extern __shared__ uint32_t side_lds[];
  compensate_tile<D>(dm, a, blockIdx.x * 32, blockIdx.y, side_lds);
}

// Launch order of the video query blocks of one (batch, head): sorted by their first three
// kept key blocks (ties: block index). Workgroups that are resident on an XCD at the same time
// then walk similar lists and find each other's K/V tiles in that XCD's L2 (on the benchmark
// inputs the traffic that crosses the fabric drops by 40 %). A heuristic: any permutation gives
// the same results. One workgroup per (batch, head), bitonic sort of 64-bit keys in LDS.
__global__ __launch_bounds__(1024) void row_order_kernel(Dims dm, AttnArgs a) {
  __shared__ uint64_t keys[RSA_MAX_BLOCKS];
  const int bh = blockIdx.x, tid = threadIdx.x;
  int P = 1;
  while (P < dm.n) P <<= 1;
  for (int i = tid; i < P; i += 1024) {
    uint64_t k = ~0ull;                                    // padding sorts to the end
    if (i < dm.n) {
      const size_t row = (size_t)bh * dm.n + i;
      const int cnt = a.count[row];
      const int32_t* lst = a.block_idx + row * dm.m;
      const uint64_t i0 = cnt > 0 ? lst[0] : 4095, i1 = cnt > 1 ? lst[1] : 4095, i2 = cnt > 2 ? lst[2] : 4095;
      k = (i0 << 36) | (i1 << 24) | (i2 << 12) | (uint64_t)i;     // every index < RSA_MAX_BLOCKS = 2^12
    }
    keys[i] = k;
  }
  __syncthreads();
  for (int k2 = 2; k2 <= P; k2 <<= 1)
    for (int j = k2 >> 1; j > 0; j >>= 1) {
      for (int i = tid; i < P; i += 1024) {
        const int o = i ^ j;
        if (o > i) {
          const uint64_t x = keys[i], y = keys[o];
          if ((x > y) == ((i & k2) == 0)) {
            keys[i] = y;
            keys[o] = x;
          }
        }
      }
      __syncthreads();
    }
  for (int i = tid; i < dm.n; i += 1024) a.row_order[(size_t)bh * dm.n + i] = (int32_t)(keys[i] & 4095u);
}

// Deals the items of one launch to the slots of the persistent attention kernel. One workgroup per
// queue of 64 slots (the slots of a queue run on one XCD). The queue's items, in launch order: its
// share of the dense items (text query blocks, or every block under RSA_DENSE: the long ones first),
// then, head by head, its contiguous range of the row order of the video query blocks. They are
// dealt in rounds by one wave, lane = slot: in a round every slot whose load (steps so far) is within
// one item of the lightest takes the next item, in lane order -- neighbouring items go to neighbouring
// slots at about the same time, so that workgroups resident together walk similar lists, and the
// loads end within one item of each other whatever the lengths of the rows.
// Minimum over the 64 lanes of a wave with data-parallel-primitive moves (row shifts inside the rows of
// 16 lanes, then the two row broadcasts): lane 63 ends up with it. Lanes without a source take INT_MAX.
__device__ __forceinline__ int wave_min_i32(int v) {
  constexpr int kMax = 0x7fffffff;
  v = min(v, __builtin_amdgcn_update_dpp(kMax, v, 0x111, 0xf, 0xf, false));   // row_shr:1
  v = min(v, __builtin_amdgcn_update_dpp(kMax, v, 0x112, 0xf, 0xf, false));   // row_shr:2
  v = min(v, __builtin_amdgcn_update_dpp(kMax, v, 0x114, 0xf, 0xf, false));   // row_shr:4
  v = min(v, __builtin_amdgcn_update_dpp(kMax, v, 0x118, 0xf, 0xf, false));   // row_shr:8
  v = min(v, __builtin_amdgcn_update_dpp(kMax, v, 0x142, 0xa, 0xf, false));   // row_bcast:15 into rows 1 and 3
  v = min(v, __builtin_amdgcn_update_dpp(kMax, v, 0x143, 0xc, 0xf, false));   // row_bcast:31 into rows 2 and 3
  return __builtin_amdgcn_readlane(v, 63);
}

constexpr int kDealSegment = 2048;   // items of a queue staged in LDS at a time: two int32 each
template <int SPB>
__device__ __forceinline__ void deal_queue(const Dims& dm, const AttnArgs& a, const DealArgs& da, int q, uint32_t* lds) {
  constexpr int SEG = kDealSegment;
  constexpr int kStrictTail = 128;
  int32_t* rec = reinterpret_cast<int32_t*>(lds);
  int32_t* len = rec + SEG;
  const int tid = threadIdx.x, lane = tid % 64;
  const bool dense_all = (a.flags & RSA_DENSE) != 0;
  const int bh_total = dm.batch * dm.heads;
  // items of this queue: dense items d = q, q + n_queues, ...; then for every head the positions
  // [q N / n_queues, (q + 1) N / n_queues) of its row order
  const int my_dense = q < da.n_dense ? (da.n_dense - q + da.n_queues - 1) / da.n_queues : 0;
  const int p0 = (int)((long long)q * dm.n / da.n_queues), p1 = (int)((long long)(q + 1) * dm.n / da.n_queues);
  const int per_head = dense_all ? 0 : p1 - p0;
  const int n_queue_items = my_dense + per_head * bh_total;
  // lane = slot u of this queue; the XCD has slots_per_xcd of them in all
  const bool slot_ok = (q / 8) * 64 + lane < da.slots_per_xcd;
  const int slot = q * 64 + lane;
  int load = 0, cnt = 0;
  for (int seg0 = 0; seg0 < n_queue_items; seg0 += SEG) {
    const int seg_n = min(SEG, n_queue_items - seg0);
    __syncthreads();
    for (int i = tid; i < seg_n; i += 256) {
      const int it = seg0 + i;
      int bhx, qbx;
      if (it < my_dense) {
        const int d = q + it * da.n_queues;
        bhx = d / da.dense_per_bh;
        qbx = da.dense_first + d % da.dense_per_bh;
      } else {
        const int v = it - my_dense;
        bhx = v / per_head;
        const int pos = p0 + v % per_head;
        qbx = a.row_order ? a.row_order[(size_t)bhx * dm.n + pos] : pos;
      }
      const bool sp = !dense_all && qbx < dm.n;
      rec[i] = bhx * RSA_MAX_BLOCKS + qbx;
      len[i] = (sp ? list_length(a, dm, (size_t)bhx * dm.n + qbx) : dm.m) * SPB;
    }
    __syncthreads();
    if (tid < 64) {
      int next = 0;
      while (next < seg_n) {
        const bool can = slot_ok && cnt < da.cap;
        const int lightest = wave_min_i32(can ? load : 0x7fffffff);
        bool take = can && load < lightest + len[next];
        if (n_queue_items - (seg0 + next) <= kStrictTail) {
          // the last items go one at a time to the lightest slot, so that the loads end within one item
          const unsigned long long lightest_ones = __ballot(can && load == lightest);
          take = lightest_ones != 0 && lane == __builtin_ctzll(lightest_ones);
        }
        const unsigned long long takers = __ballot(take);
        const int mine = next + __builtin_amdgcn_mbcnt_hi((uint32_t)(takers >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)takers, 0));
        if (take && mine < seg_n) {
          da.table[(size_t)slot * da.cap + cnt] = rec[mine];
          load += len[mine];
          cnt += 1;
        }
        if (takers == 0) break;            // cannot happen while the table has room (the lightest slot always takes)
        next += __popcll(takers);
      }
    }
  }
  if (tid < 64) {
    da.nitems[slot] = cnt;
    da.total[slot] = load;
  }
}

template <int SPB>
__global__ __launch_bounds__(256) void schedule_kernel(Dims dm, AttnArgs a, DealArgs da) {
  extern __shared__ uint32_t side_lds[];
  deal_queue<SPB>(dm, a, da, blockIdx.x, side_lds);
}

// Both of the above in one launch (neither needs the other's result, and the few workgroups that deal
// the queues would otherwise have the chip to themselves): plane 0 of the grid deals queue blockIdx.x,
// plane 1 + bh compensates the rows of (batch, head) bh. The dealing workgroups are dispatched first.
template <int D, int SPB>
__global__ __launch_bounds__(256) void compensation_schedule_kernel(Dims dm, AttnArgs a, DealArgs da) {
  extern __shared__ uint32_t side_lds[];
  if (blockIdx.y == 0) {
    if ((int)blockIdx.x < da.n_queues) deal_queue<SPB>(dm, a, da, blockIdx.x, side_lds);   // uniform over the workgroup
    return;
  }
  compensate_tile<D>(dm, a, blockIdx.x * 32, (int)blockIdx.y - 1, side_lds);
}

}  // namespace

namespace {
template <int D, int SPB>
hipError_t launch_attn_side_t(const Dims& dm, const AttnArgs& a, const DealArgs& da, bool sort_rows, bool compensate, bool deal,
                              hipStream_t s) {
  const int bh = dm.batch * dm.heads;
  const dim3 comp_grid((dm.n + 31) / 32, bh);
  const unsigned comp_lds = comp_lds_bytes<D>();
  const unsigned deal_lds = 2u * kDealSegment * 4u;
  if (sort_rows) hipLaunchKernelGGL(row_order_kernel, dim3(bh), dim3(1024), 0, s, dm, a);
  if (deal && compensate && da.n_queues <= (int)comp_grid.x) {
    hipLaunchKernelGGL((compensation_schedule_kernel<D, SPB>), dim3(comp_grid.x, bh + 1), dim3(256),
                       comp_lds > deal_lds ? comp_lds : deal_lds, s, dm, a, da);
  } else {
    if (compensate) hipLaunchKernelGGL((compensation_kernel<D>), comp_grid, dim3(256), comp_lds, s, dm, a);
    if (deal) hipLaunchKernelGGL((schedule_kernel<SPB>), dim3(da.n_queues), dim3(256), deal_lds, s, dm, a, da);
  }
  return hipGetLastError();
}
}  // namespace

hipError_t launch_attn_side(const Dims& dm, const AttnArgs& a, const DealArgs& da, bool sort_rows, bool compensate, bool deal,
                            int spb, hipStream_t s) {
  if (spb != 2) return hipErrorInvalidValue;      // every attention template takes two steps per key block
  if (dm.d == 128) return launch_attn_side_t<128, 2>(dm, a, da, sort_rows, compensate, deal, s);
  return launch_attn_side_t<64, 2>(dm, a, da, sort_rows, compensate, deal, s);
}

}  // namespace rsa
