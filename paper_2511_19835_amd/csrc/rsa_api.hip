// C-ABI entry points of librsa.so: host-side validation, workspace carving, launches.
#include <math.h>

#include <atomic>

#include "rsa_common.hpp"

namespace {

using rsa::Dims;

int make_dims(const rsa_shape* sh, Dims* out) {
  if (!sh) return RSA_E_NULL;
  if (sh->batch < 1 || sh->heads < 1 || sh->t_video < 1 || sh->t_text < 0) return RSA_E_SHAPE;
  if (sh->head_dim != 64 && sh->head_dim != 128) return RSA_E_UNSUPPORTED;
  if (sh->block != 64 && sh->block != 128) return RSA_E_UNSUPPORTED;
  if (sh->stride_t < sh->head_dim || sh->stride_b < 1 || sh->stride_h < 1) return RSA_E_SHAPE;
  if ((sh->stride_t % 8) || (sh->stride_b % 8) || (sh->stride_h % 8)) return RSA_E_SHAPE;
  // the kernels address the rows of one key block with 32-bit byte offsets
  if ((int64_t)sh->block * sh->stride_t * 2 >= ((int64_t)1 << 31)) return RSA_E_UNSUPPORTED;
  if (!(sh->scale >= 0.f) || !isfinite(sh->scale)) return RSA_E_RANGE;
  Dims d;
  d.batch = sh->batch;
  d.heads = sh->heads;
  d.d = sh->head_dim;
  d.blk = sh->block;
  d.tv = sh->t_video;
  d.tt = sh->t_text;
  d.t = d.tv + d.tt;
  int64_t n = (d.tv + d.blk - 1) / d.blk;
  int64_t mt = (d.tt + d.blk - 1) / d.blk;
  if (n + mt > RSA_MAX_BLOCKS) return RSA_E_UNSUPPORTED;
  if ((int64_t)d.batch * d.heads > 65535) return RSA_E_UNSUPPORTED;
  d.n = (int)n;
  d.mt = (int)mt;
  d.m = (int)(n + mt);
  d.w = (d.m + 31) / 32;
  d.sb = sh->stride_b;
  d.sh = sh->stride_h;
  d.st = sh->stride_t;
  d.scale = sh->scale > 0.f ? sh->scale : 1.0f / sqrtf((float)d.d);
  *out = d;
  return RSA_OK;
}

inline size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }

// Carving of the pooling workspace; every piece 256-byte aligned.
struct PoolWs {
  size_t qpb, kpb, dbt, total;
};
PoolWs pool_ws_layout(const Dims& d) {
  size_t bh = (size_t)d.batch * d.heads;
  PoolWs w;
  size_t off = 0;
  w.qpb = off; off += align256(bh * rsa::gate_operand_vectors(d.n) * d.d * sizeof(uint16_t));
  w.kpb = off; off += align256(bh * rsa::gate_operand_vectors(d.m) * d.d * sizeof(uint16_t));
  w.dbt = off;  off += align256(bh * (size_t)d.n * d.m * sizeof(float));
  w.total = off;
  return w;
}

// rsa_sparse_attn_rectified scratch: the pooled compensation term C_n, fp32 [b][h][N][d]; the launch
// order of the video query blocks, int32 [b][h][N]; the schedule of the persistent kernel (item
// table, items and steps per slot).
struct AttnWs {
  size_t comp, order, table, nitems, total, bytes;
  size_t table_entries;
};
AttnWs attn_ws_layout(const Dims& d) {
  AttnWs w;
  size_t off = 0;
  w.comp = off;   off += align256((size_t)d.batch * d.heads * d.n * d.d * sizeof(float));
  w.order = off;  off += align256((size_t)d.batch * d.heads * d.n * sizeof(int32_t));
  w.table_entries = rsa::attn_sched_entries(d);
  w.table = off;  off += align256(w.table_entries * sizeof(int32_t));
  w.nitems = off; off += align256(RSA_ATTN_SCHED_SLOTS * sizeof(int32_t));
  w.total = off;  off += align256(RSA_ATTN_SCHED_SLOTS * sizeof(int32_t));
  w.bytes = off;
  return w;
}
size_t attn_ws_size(const Dims& d) { return attn_ws_layout(d).bytes; }

// Workgroups of the persistent attention kernel: one per CU of the current device, in whole
// multiples of the 8 XCDs, at most RSA_ATTN_MAX_WGS. The CU count is read once per device.
constexpr int kMaxDevices = 64;
std::atomic<int> g_cu_count[kMaxDevices];
int attn_workgroups() {
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return 0;
  int cus = g_cu_count[dev].load(std::memory_order_acquire);
  if (cus == 0) {
    if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus < 8) return 0;
    g_cu_count[dev].store(cus, std::memory_order_release);
  }
  int n = cus < RSA_ATTN_MAX_WGS ? cus : RSA_ATTN_MAX_WGS;
  return n - n % 8;
}

// Argument checks shared by the two attention entry points. RSA_DENSE drops the other flags.
int check_attn_args(const Dims&, const void* Q, const void* K, const void* Vt, const int32_t* block_idx,
                    const int32_t* count, const uint32_t* mask_bits, const float* R, const float* Apool,
                    const uint32_t* Mc_bits, const float* Vp, int* flags, const void* O) {
  if (*flags & ~(RSA_RECTIFY_CRITICAL | RSA_COMPENSATE | RSA_DENSE)) return RSA_E_RANGE;
  if (!Q || !K || !Vt || !O) return RSA_E_NULL;
  if (*flags & RSA_DENSE) {
    *flags = RSA_DENSE;
    return RSA_OK;
  }
  if (!block_idx || !count) return RSA_E_NULL;
  if ((*flags & RSA_RECTIFY_CRITICAL) && !R) return RSA_E_NULL;
  if ((*flags & RSA_COMPENSATE) && (!mask_bits || !Apool || !Mc_bits || !Vp)) return RSA_E_NULL;
  return RSA_OK;
}

// `ws` (may be NULL without RSA_COMPENSATE): C_n, then the launch order of the video query blocks.
int enqueue_attn(const Dims& d, const void* Q, const void* K, const void* Vt, const int32_t* block_idx,
                 const int32_t* count, const uint32_t* mask_bits, const float* R, const float* Apool,
                 const uint32_t* Mc_bits, const float* Vp, int flags, void* O, float* lse, void* ws, void* stream) {
  rsa::AttnArgs aa;
  aa.Q = (const uint16_t*)Q; aa.K = (const uint16_t*)K; aa.Vt = (const uint16_t*)Vt;
  aa.block_idx = block_idx; aa.count = count; aa.mask_bits = mask_bits; aa.Mc_bits = Mc_bits;
  aa.R = R; aa.Apool = Apool; aa.Vp = Vp; aa.O = (uint16_t*)O; aa.lse = lse;
  aa.flags = flags;
  rsa::AttnSched sch = {};
  sch.n_wg = attn_workgroups();
  if (sch.n_wg < 8) return RSA_E_LAUNCH;
  char* wsb = (char*)ws;
  const AttnWs wl = attn_ws_layout(d);
  aa.comp = ws ? (float*)(wsb + wl.comp) : nullptr;
  aa.row_order = (ws && !(flags & RSA_DENSE)) ? (int32_t*)(wsb + wl.order) : nullptr;
  if (ws) {
    sch.table = (int32_t*)(wsb + wl.table);
    sch.nitems = (int32_t*)(wsb + wl.nitems);
    sch.total = (int32_t*)(wsb + wl.total);
    sch.table_entries = wl.table_entries;
  }
  if (rsa::launch_attn(d, aa, sch, (hipStream_t)stream) != hipSuccess) return RSA_E_LAUNCH;
  return RSA_OK;
}

// Scratch of rsa_sparse_attn_rectified_static: one array per GPU, held from the moment the library's
// code object is loaded on that GPU until the process ends. In host code the array's name is only a
// handle for hipGetSymbolAddress; the device address it yields (one per device) is what kernels get.
__attribute__((used)) static __device__ __align__(256) unsigned char scratch[RSA_STATIC_SCRATCH_BYTES];

std::atomic<void*> g_scratch_ptr[kMaxDevices];

void* static_scratch_of_current_device() {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return nullptr;
  void* p = g_scratch_ptr[dev].load(std::memory_order_acquire);
  if (p) return p;
  // first call on this device (racing first calls all get the same answer)
  if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return nullptr;
  g_scratch_ptr[dev].store(p, std::memory_order_release);
  return p;
}

}  // namespace

extern "C" {

int rsa_block_counts(const rsa_shape* shape, int64_t* n_video_blocks, int64_t* n_blocks,
                     int64_t* mask_words) {
  Dims d;
  int rc = make_dims(shape, &d);
  if (rc != RSA_OK) return rc;
  if (n_video_blocks) *n_video_blocks = d.n;
  if (n_blocks) *n_blocks = d.m;
  if (mask_words) *mask_words = d.w;
  return RSA_OK;
}

int rsa_workspace_bytes(const rsa_shape* shape, size_t* pool_ws_bytes, size_t* attn_ws_bytes) {
  Dims d;
  int rc = make_dims(shape, &d);
  if (rc != RSA_OK) return rc;
  if (pool_ws_bytes) *pool_ws_bytes = pool_ws_layout(d).total;
  if (attn_ws_bytes) *attn_ws_bytes = attn_ws_size(d);
  return RSA_OK;
}

int rsa_pool(const rsa_shape* shape, const void* Q, const void* K, const void* V, float* Qp,
             float* Kp, float* Vp, void* Vt, float* Spool, float* Apool, float* Lmass,
             uint32_t* Mc_bits, int gapr_mode, void* ws, size_t ws_bytes, void* stream) {
  Dims d;
  int rc = make_dims(shape, &d);
  if (rc != RSA_OK) return rc;
  if (!Q || !K || !V || !Qp || !Kp || !Vp || !Vt || !Spool || !Apool || !Lmass || !Mc_bits)
    return RSA_E_NULL;
  if (gapr_mode < 0 || gapr_mode > 2) return RSA_E_RANGE;
  PoolWs wl = pool_ws_layout(d);
  if (!ws) return RSA_E_NULL;
  if (ws_bytes < wl.total || ((uintptr_t)ws & 255)) return RSA_E_WORKSPACE;
  hipStream_t s = (hipStream_t)stream;
  char* wsb = (char*)ws;

  rsa::PoolArgs pa;
  pa.Q = (const uint16_t*)Q; pa.K = (const uint16_t*)K; pa.V = (const uint16_t*)V;
  pa.Qp = Qp; pa.Kp = Kp; pa.Vp = Vp; pa.Vt = (uint16_t*)Vt;
  pa.Qpb = (uint16_t*)(wsb + wl.qpb);
  pa.Kpb = (uint16_t*)(wsb + wl.kpb);
  // with the gate on, the launch that reads the key blocks for their deviations pools them as well
  pa.skip_k = gapr_mode == 1;
  pa.text_K = (const uint16_t*)K; pa.text_Lmass = Lmass;     // the text log-masses ride with the pooling of V
  if (rsa::launch_pool(d, pa, s) != hipSuccess) return RSA_E_LAUNCH;

  rsa::GaprArgs ga;
  ga.Q = (const uint16_t*)Q; ga.K = (const uint16_t*)K;
  ga.Qp = Qp; ga.Kp = Kp;
  ga.Qpb = pa.Qpb; ga.Kpb = pa.Kpb; ga.Spool = Spool;
  ga.DBt = (float*)(wsb + wl.dbt);
  ga.Mc_bits = Mc_bits; ga.mode = gapr_mode;
  if (gapr_mode == 1) {
    ga.Kp_out = Kp; ga.Kpb_out = pa.Kpb;
    if (rsa::launch_gapr_keys(d, ga, s) != hipSuccess) return RSA_E_LAUNCH;
  }

  rsa::ScoreArgs sa;
  sa.K = (const uint16_t*)K; sa.Qp = Qp; sa.Kp = Kp;
  sa.Spool = Spool; sa.Apool = Apool; sa.Lmass = Lmass;
  sa.text_done = true;
  if (rsa::launch_scores(d, sa, s) != hipSuccess) return RSA_E_LAUNCH;

  if (gapr_mode == 1) {
    if (rsa::launch_gapr_queries(d, ga, s) != hipSuccess) return RSA_E_LAUNCH;
    return RSA_OK;
  }
  if (rsa::launch_gapr(d, ga, s) != hipSuccess) return RSA_E_LAUNCH;
  return RSA_OK;
}

int rsa_pool_values(const rsa_shape* shape, const void* V, float* Vp, void* Vt, void* stream) {
  Dims d;
  int rc = make_dims(shape, &d);
  if (rc != RSA_OK) return rc;
  if (!V || !Vp || !Vt) return RSA_E_NULL;
  rsa::PoolArgs pa = {};
  pa.V = (const uint16_t*)V; pa.Vp = Vp; pa.Vt = (uint16_t*)Vt;
  if (rsa::launch_pool(d, pa, (hipStream_t)stream) != hipSuccess) return RSA_E_LAUNCH;
  return RSA_OK;
}

int rsa_implicit_attention(const rsa_shape* shape, const void* K, const float* Qp, const float* Kp,
                           float* Spool, float* Lmass, float* Apool, void* stream) {
  Dims d;
  int rc = make_dims(shape, &d);
  if (rc != RSA_OK) return rc;
  if (!K || !Qp || !Kp || !Spool || !Lmass || !Apool) return RSA_E_NULL;
  rsa::ScoreArgs sa;
  sa.K = (const uint16_t*)K; sa.Qp = Qp; sa.Kp = Kp;
  sa.Spool = Spool; sa.Apool = Apool; sa.Lmass = Lmass;
  if (rsa::launch_scores(d, sa, (hipStream_t)stream) != hipSuccess) return RSA_E_LAUNCH;
  return RSA_OK;
}

int rsa_select_blocks(const rsa_shape* shape, const float* Lmass, const float* Apool,
                      double sparsity, double p, const uint32_t* forced_bits,
                      uint32_t* mask_bits, int32_t* block_idx, int32_t* count, float* R,
                      void* stream) {
  Dims d;
  int rc = make_dims(shape, &d);
  if (rc != RSA_OK) return rc;
  if (!Lmass || !Apool || !mask_bits || !block_idx || !count || !R) return RSA_E_NULL;
  if (!(sparsity >= 0.0 && sparsity <= 1.0) || !(p >= 0.0 && p <= 1.0)) return RSA_E_RANGE;
  int64_t keep = (int64_t)d.m - (int64_t)floor(sparsity * (double)d.m + 1e-6);
  if (keep < 1) keep = 1;
  if (keep > d.m) keep = d.m;
  rsa::SelectArgs sa;
  sa.Lmass = Lmass; sa.Apool = Apool; sa.forced = forced_bits;
  sa.mask_bits = mask_bits; sa.block_idx = block_idx; sa.count = count; sa.R = R;
  sa.keep = (int)keep; sa.p = (float)p;
  if (rsa::launch_select(d, sa, (hipStream_t)stream) != hipSuccess) return RSA_E_LAUNCH;
  return RSA_OK;
}

int rsa_adjacency_mask(const rsa_shape* shape, const int32_t* grid, const int32_t* tile, int radius,
                       uint32_t* forced_bits, void* stream) {
  Dims d;
  int rc = make_dims(shape, &d);
  if (rc != RSA_OK) return rc;
  if (!grid || !tile || !forced_bits) return RSA_E_NULL;
  for (int i = 0; i < 3; ++i)
    if (grid[i] < 1 || tile[i] < 1) return RSA_E_SHAPE;
  if ((int64_t)grid[0] * grid[1] * grid[2] != d.tv) return RSA_E_SHAPE;
  if (radius < 0 || radius > 64) return RSA_E_RANGE;
  if (rsa::launch_adjacency(d, grid, tile, radius, forced_bits, (hipStream_t)stream) != hipSuccess) return RSA_E_LAUNCH;
  return RSA_OK;
}

int rsa_reorder_tokens(const rsa_shape* shape, const int32_t* grid, const int32_t* tile, int direction,
                       const void* src, void* dst, void* stream) {
  Dims d;
  int rc = make_dims(shape, &d);
  if (rc != RSA_OK) return rc;
  if (!grid || !tile || !src || !dst) return RSA_E_NULL;
  for (int i = 0; i < 3; ++i)
    if (grid[i] < 1 || tile[i] < 1) return RSA_E_SHAPE;
  if ((int64_t)grid[0] * grid[1] * grid[2] != d.tv) return RSA_E_SHAPE;
  if ((direction != 0 && direction != 1) || src == dst) return RSA_E_RANGE;
  if (rsa::launch_reorder(d, grid, tile, direction, (const uint16_t*)src, (uint16_t*)dst, (hipStream_t)stream) !=
      hipSuccess)
    return RSA_E_LAUNCH;
  return RSA_OK;
}

int rsa_sparse_attn_rectified(const rsa_shape* shape, const void* Q, const void* K, const void* Vt,
                              const int32_t* block_idx, const int32_t* count,
                              const uint32_t* mask_bits, const float* R, const float* Apool,
                              const uint32_t* Mc_bits, const float* Vp, int flags, void* O,
                              float* lse, void* ws, size_t ws_bytes, void* stream) {
  Dims d;
  int rc = make_dims(shape, &d);
  if (rc != RSA_OK) return rc;
  rc = check_attn_args(d, Q, K, Vt, block_idx, count, mask_bits, R, Apool, Mc_bits, Vp, &flags, O);
  if (rc != RSA_OK) return rc;
  if (!(flags & RSA_DENSE)) {
    if ((flags & RSA_COMPENSATE) && !ws) return RSA_E_NULL;
    if (ws && (ws_bytes < attn_ws_size(d) || ((uintptr_t)ws & 255))) return RSA_E_WORKSPACE;
  } else if (ws && (ws_bytes < attn_ws_size(d) || ((uintptr_t)ws & 255))) {
    ws = nullptr;            // a dense launch never needed a workspace: without a usable one it runs in index order
  }
  return enqueue_attn(d, Q, K, Vt, block_idx, count, mask_bits, R, Apool, Mc_bits, Vp, flags, O, lse, ws, stream);
}

int rsa_sparse_attn_rectified_static(const rsa_shape* shape, const void* Q, const void* K, const void* Vt,
                                     const int32_t* block_idx, const int32_t* count,
                                     const uint32_t* mask_bits, const float* R, const float* Apool,
                                     const uint32_t* Mc_bits, const float* Vp, int flags, void* O,
                                     float* lse, void* stream) {
  Dims d;
  int rc = make_dims(shape, &d);
  if (rc != RSA_OK) return rc;
  rc = check_attn_args(d, Q, K, Vt, block_idx, count, mask_bits, R, Apool, Mc_bits, Vp, &flags, O);
  if (rc != RSA_OK) return rc;
  void* ws = nullptr;
  if (!(flags & RSA_DENSE)) {
    if (attn_ws_size(d) > (size_t)RSA_STATIC_SCRATCH_BYTES) return RSA_E_WORKSPACE;
    ws = static_scratch_of_current_device();
    if (!ws) return RSA_E_LAUNCH;
  }
  return enqueue_attn(d, Q, K, Vt, block_idx, count, mask_bits, R, Apool, Mc_bits, Vp, flags, O, lse, ws, stream);
}

const char* rsa_status_string(int status) {
  switch (status) {
    case RSA_OK: return "ok";
    case RSA_E_NULL: return "a required pointer is NULL";
    case RSA_E_SHAPE: return "invalid shape or strides";
    case RSA_E_UNSUPPORTED: return "unsupported head_dim / block / block count";
    case RSA_E_WORKSPACE: return "workspace too small or misaligned";
    case RSA_E_RANGE: return "argument out of range";
    case RSA_E_LAUNCH: return "HIP launch failed";
    default: return "unknown status";
  }
}

}  // extern "C"
