// What the attention launch and the small kernels that run before it share: the shape of the schedule
// (host and device agree on it), the arguments of the dealing kernel, and the one launcher of those kernels.
#pragma once
#include "rsa_common.hpp"

namespace rsa {

// Entries of a video query block's list as every kernel here takes them: the count that
// rsa_select_blocks wrote, held to 1 .. M so that no count, whatever it is, can derail the loops.
__device__ __forceinline__ int list_length(const AttnArgs& a, const Dims& dm, size_t vrow) {
  typedef const int32_t __attribute__((address_space(4))) * const_i32_t;     // scalar loads
  const int c = ((const_i32_t)(uintptr_t)a.count)[vrow];
  return min(max(c, 1), dm.m);
}

struct DealArgs {
  int32_t* table;           // [queues * 64][cap]
  int32_t* nitems;          // [queues * 64]
  int32_t* total;           // [queues * 64]
  int cap, n_queues, slots_per_xcd;
  int n_dense, dense_per_bh, dense_first;
};

// Sizes of the schedule for `n_wg` resident workgroups of NGRP groups (host and launcher agree on them).
struct SchedShape {
  int n_queues, slots_per_xcd, cap, chunk, n_items, n_dense, dense_per_bh, dense_first;
};
inline SchedShape sched_shape(const Dims& dm, int flags, int n_wg, int ngrp) {
  SchedShape s;
  const bool dense_all = (flags & RSA_DENSE) != 0;
  const int bh = dm.batch * dm.heads;
  s.slots_per_xcd = (n_wg / 8) * ngrp;
  s.n_queues = 8 * ((s.slots_per_xcd + 63) / 64);
  s.dense_per_bh = dense_all ? dm.m : dm.mt;
  s.dense_first = dense_all ? 0 : dm.n;
  s.n_dense = bh * s.dense_per_bh;
  s.n_items = s.n_dense + (dense_all ? 0 : bh * dm.n);
  s.chunk = (dm.n + s.n_queues - 1) / s.n_queues;
  const long long longest = (s.n_dense + s.n_queues - 1) / s.n_queues + (dense_all ? 0LL : (long long)bh * s.chunk);
  // room for twice the average share of a slot, so that a queue of very unequal items still balances;
  // the last queue of an XCD may have fewer than 64 slots
  const int fewest = s.slots_per_xcd % 64 ? s.slots_per_xcd % 64 : 64;
  s.cap = (int)(2 * ((longest + fewest - 1) / fewest) + 8);
  return s;
}

// Launches, on stream s and in this order, the sort of the launch order (when `sort_rows`: writes a.row_order), the
// pooled compensation (when `compensate`) and the dealing of the schedule (when `deal`; da filled by the
// caller) -- the last two as one launch when both are wanted and the grid allows it. d = head dimension,
// spb = steps per key block of the attention kernel that will read the table.
hipError_t launch_attn_side(const Dims& dm, const AttnArgs& a, const DealArgs& da, bool sort_rows, bool compensate, bool deal,
                            int spb, hipStream_t s);

}  // namespace rsa
