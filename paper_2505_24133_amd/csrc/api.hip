// C ABI of librkv: argument validation, workspace carve-up and kernel sequencing.
// Nothing here touches device memory from the host or synchronises the stream.
#include <math.h>

#include <algorithm>
#include <atomic>

#include "rkv_internal.h"

namespace rkv {

// Compute units of the current device, queried once per device ordinal and kept (256, the MI355X, when
// no device is present: host-only use of the size query).
int device_compute_units() {
  constexpr int kMaxDevices = 64;
  static std::atomic<int> cached[kMaxDevices];          // 0 = not asked yet
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) {
    (void)hipGetLastError();
    return 256;
  }
  int cus = cached[dev].load(std::memory_order_relaxed);
  if (cus > 0) return cus;
  if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus < 1) {
    (void)hipGetLastError();
    cus = 256;
  }
  cached[dev].store(cus, std::memory_order_relaxed);
  return cus;
}

static constexpr uint32_t kGqaFlags = RKV_FLAG_GQA_SOFTMAX_THEN_MAX | RKV_FLAG_GQA_SOFTMAX_THEN_MEAN;
static constexpr uint32_t kKnownFlags =
    RKV_FLAG_SKIP_SATURATED | RKV_FLAG_POOL_AFTER_MEAN | RKV_FLAG_SHARED_SELECTION | kGqaFlags |
    RKV_FLAG_RECENCY_TRANSPOSED | RKV_FLAG_TRIANGULAR_SCAN;

static size_t align_up(size_t x) { return (x + 255) & ~(size_t)255; }

rkv_status make_plan(const rkv_params* prm, Plan* pl) {
  if (prm == nullptr) return RKV_ERR_NULL;
  const rkv_params& q = *prm;
  if (q.num_problems < 0 || q.kv_heads < 1 || q.q_heads < 1 || q.alpha < 1 || q.n_tokens < 1 || q.budget < 1)
    return RKV_ERR_SHAPE;
  if (q.q_heads % q.kv_heads != 0) return RKV_ERR_SHAPE;
  if (q.n_tokens <= q.alpha || q.budget <= q.alpha) return RKV_ERR_SHAPE;
  if (q.head_dim != kHeadDim || (q.flags & ~kKnownFlags) != 0) return RKV_ERR_UNSUPPORTED;
  const int G = q.q_heads / q.kv_heads;
  if (q.alpha > kMaxQRows || (int64_t)G * q.alpha > kMaxQRows || q.n_tokens > 32768) return RKV_ERR_UNSUPPORTED;
  if ((int64_t)q.num_problems * q.kv_heads > (1 << 22)) return RKV_ERR_UNSUPPORTED;
  if (!(q.lambda >= 0.f && q.lambda <= 1.f) || !(q.sim_threshold >= 0.f && q.sim_threshold <= 1.f) ||
      !(q.eps > 0.f) || !isfinite(q.eps) || q.beta < 0 || q.pool_w < 0 || (q.flags & kGqaFlags) == kGqaFlags)
    return RKV_ERR_PARAM;
  if ((q.flags & RKV_FLAG_TRIANGULAR_SCAN) != 0 &&
      (q.beta != 1 || (q.flags & (RKV_FLAG_RECENCY_TRANSPOSED | RKV_FLAG_SKIP_SATURATED)) != 0))
    return RKV_ERR_PARAM;
  const int64_t pool_rows = q.alpha + ((q.flags & RKV_FLAG_POOL_AFTER_MEAN) ? 1 : 0);
  if (pool_rows * (q.pool_w > 0 ? 2 * (int64_t)q.pool_w : 1) > 16384 || q.pool_w > 1000) return RKV_ERR_UNSUPPORTED;

  pl->P = q.num_problems; pl->H = q.kv_heads; pl->G = G; pl->N = q.n_tokens; pl->alpha = q.alpha;
  pl->n = q.n_tokens - q.alpha; pl->budget = q.budget; pl->k_sel = q.budget - q.alpha;
  pl->W = q.pool_w; pl->beta = q.beta; pl->T = q.sim_threshold; pl->lambda = q.lambda; pl->eps = q.eps;
  pl->skip_saturated = (q.flags & RKV_FLAG_SKIP_SATURATED) != 0;
  pl->pool_after_mean = (q.flags & RKV_FLAG_POOL_AFTER_MEAN) != 0;
  pl->shared_selection = (q.flags & RKV_FLAG_SHARED_SELECTION) != 0;
  pl->recency_transposed = (q.flags & RKV_FLAG_RECENCY_TRANSPOSED) != 0;
  pl->triangular = (q.flags & RKV_FLAG_TRIANGULAR_SCAN) != 0;
  pl->gqa_mode = (q.flags & RKV_FLAG_GQA_SOFTMAX_THEN_MAX) ? 1 : ((q.flags & RKV_FLAG_GQA_SOFTMAX_THEN_MEAN) ? 2 : 0);
  pl->qrows = (pl->gqa_mode == 0) ? q.alpha : G * q.alpha;
  pl->heads = q.num_problems * q.kv_heads;
  pl->chunks = (pl->n + kChunk - 1) / kChunk;
  pl->n_pad = pl->chunks * kChunk;

  pl->paged = q.page_size != 0;
  pl->page_shift = 0; pl->table_stride = q.table_stride; pl->block_table = q.block_table;
  pl->kspage = q.k_stride_page; pl->vspage = q.v_stride_page;
  if (pl->paged) {
    if (q.page_size != 16 && q.page_size != 32 && q.page_size != 64 && q.page_size != 128) return RKV_ERR_UNSUPPORTED;
    while ((1 << pl->page_shift) < q.page_size) ++pl->page_shift;
    if (q.num_problems > 0 && q.block_table == nullptr) return RKV_ERR_NULL;
    if ((int64_t)q.table_stride * q.page_size < q.n_tokens) return RKV_ERR_SHAPE;
    auto ok = [](int64_t s) { return s > 0 && (s % 8) == 0; };
    if (!ok(q.k_stride_page) || !ok(q.v_stride_page) || !ok(q.k_stride_token) || !ok(q.v_stride_token) ||
        q.k_stride_token < kHeadDim || q.v_stride_token < kHeadDim || q.k_stride_token > 32768 || q.v_stride_token > 32768 ||
        q.k_stride_head < 0 || q.v_stride_head < 0 || (q.k_stride_head % 8) != 0 || (q.v_stride_head % 8) != 0 ||
        (q.kv_heads > 1 && (q.k_stride_head == 0 || q.v_stride_head == 0)))
      return RKV_ERR_SHAPE;
  }
  auto strides = [&](int64_t sp, int64_t sh, int64_t st, int64_t* op, int64_t* oh, int64_t* ot) -> bool {
    if (pl->paged && op != &pl->osp) {                   // validated above; the problem stride is unused
      *op = 0; *oh = sh; *ot = st;
      return true;
    }
    if (sp == 0 && sh == 0 && st == 0) {
      *ot = kHeadDim; *oh = (int64_t)q.n_tokens * kHeadDim; *op = *oh * q.kv_heads;
      return true;
    }
    if (st < kHeadDim || st > 32768 || (st % 8) != 0 || (sh % 8) != 0 || (sp % 8) != 0 || sh < 0 || sp < 0) return false;
    if (q.kv_heads > 1 && sh == 0) return false;
    if (q.num_problems > 1 && sp == 0) return false;
    *op = sp; *oh = sh; *ot = st;
    return true;
  };
  if (!strides(q.k_stride_problem, q.k_stride_head, q.k_stride_token, &pl->ksp, &pl->ksh, &pl->kst)) return RKV_ERR_SHAPE;
  if (!strides(q.v_stride_problem, q.v_stride_head, q.v_stride_token, &pl->vsp, &pl->vsh, &pl->vst)) return RKV_ERR_SHAPE;
  // observation queries [P, q_heads, alpha, d]: 0,0,0 = dense; otherwise rows 16-byte aligned, slots of a
  // head and heads of a problem apart by the given strides
  if (q.q_stride_problem == 0 && q.q_stride_head == 0 && q.q_stride_token == 0) {
    pl->qst = kHeadDim; pl->qsh = (int64_t)q.alpha * kHeadDim; pl->qsp = pl->qsh * q.q_heads;
  } else {
    const int64_t st = q.q_stride_token, sh = q.q_stride_head, sp = q.q_stride_problem;
    if (st < kHeadDim || (st % 8) != 0 || (sh % 8) != 0 || (sp % 8) != 0 || sh < 0 || sp < 0) return RKV_ERR_SHAPE;
    if (q.q_heads > 1 && sh == 0) return RKV_ERR_SHAPE;
    if (q.num_problems > 1 && sp == 0) return RKV_ERR_SHAPE;
    pl->qst = st; pl->qsh = sh; pl->qsp = sp;
  }
  if (q.o_stride_problem == 0 && q.o_stride_head == 0 && q.o_stride_token == 0) {
    pl->ost = kHeadDim; pl->osh = (int64_t)q.budget * kHeadDim; pl->osp = pl->osh * q.kv_heads;
  } else {
    if (!strides(q.o_stride_problem, q.o_stride_head, q.o_stride_token, &pl->osp, &pl->osh, &pl->ost)) return RKV_ERR_SHAPE;
  }

  // ---- how the similarity pass is cut into workgroups (two are resident per compute unit): when the
  // row blocks of all heads would leave most of the machine idle, the column scan of every row block
  // is split over several workgroups.  The workspace is sized for the largest split any device could
  // choose (parts_reserved), so the size query does not depend on the device that is current.
  int parts_reserved = 1;
  {
    // (counted in row blocks of the dense kernel also for RKV_FLAG_SKIP_SATURATED, whose own row blocks are
    // smaller: the two must take the same decision, because the split changes the order of the last few
    // floating-point operations and the flag promises bit-identical results)
    const int64_t blocks = (int64_t)pl->heads * ((pl->n + kGramRows - 1) / kGramRows);
    const int nct = (pl->n + kGramTile - 1) / kGramTile;
    pl->gram_parts = 1;
    if (pl->beta == 1 && !pl->recency_transposed && !pl->triangular && blocks > 0 && blocks <= kGramSplitMaxBlocks) {
      parts_reserved = std::min(nct, kGramMaxParts);
      const int64_t slots = 2 * (int64_t)device_compute_units();
      if (blocks <= slots / 2)
        pl->gram_parts = (int)std::max<int64_t>(1, std::min<int64_t>(parts_reserved, slots / blocks));
    }
  }

  size_t off = 0;
  const size_t heads = (size_t)pl->heads, np = (size_t)pl->n_pad;
  auto take = [&](size_t bytes) { const size_t o = off; off = align_up(off + bytes); return o; };
  pl->off_rnorm = take(heads * np * 4);
  pl->off_upart = take(heads * pl->chunks * kHeadDim * 4);
  pl->off_logit = take(heads * pl->qrows * np * 4);
  pl->off_stats = take(heads * pl->chunks * 4 * pl->qrows * 2 * 4);
  pl->off_sbar = take(heads * np * 4);
  pl->off_imp = take(heads * np * 4);
  pl->off_red = take(heads * np * 4);
  pl->off_z = take(heads * np * 4);
  pl->off_credit = take(pl->recency_transposed || pl->triangular ? heads * np * 8 : 0);
  const size_t parts = (size_t)parts_reserved;
  const bool reports = parts > 1 || pl->triangular;          // per-row reports merged by the finalize kernel
  pl->off_pcnt = take(reports ? heads * parts * np * 4 : 0);
  pl->off_ppre = take(reports ? heads * parts * np * 4 : 0);
  pl->off_kdense = take(pl->paged ? heads * np * kHeadDim * 2 : 0);
  pl->off_idx = take(heads * (size_t)pl->budget * 4);
  pl->total = off;
  return RKV_OK;
}

static rkv_status check_ws(const Plan& pl, const void* ws, size_t ws_bytes) {
  if (pl.total == 0) return RKV_OK;     // empty batch: no scratch needed
  if (ws == nullptr || ((uintptr_t)ws & 255) != 0 || ws_bytes < pl.total) return RKV_ERR_WORKSPACE;
  return RKV_OK;
}

static rkv_status hip_status(hipError_t e) { return e == hipSuccess ? RKV_OK : RKV_ERR_HIP; }

// Scratch of rkv_compress_static: one array per GPU, held from the moment the library's code is loaded on
// that GPU until the process ends.  In host code the array's name is only a handle for
// hipGetSymbolAddress; the address kernels and copies use is looked up once per device and kept.
static __device__ __align__(256) unsigned char scratch[RKV_STATIC_SCRATCH_BYTES];

static rkv_status static_scratch(char** out) {
  constexpr int kMaxDevices = 64;
  static std::atomic<void*> address[kMaxDevices];       // nullptr = not looked up yet on that device
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) {
    (void)hipGetLastError();
    return RKV_ERR_HIP;
  }
  void* p = address[dev].load(std::memory_order_acquire);
  if (p == nullptr) {
    // with device `dev` current this returns the address of that device's copy of the array; two threads
    // racing here look up the same value
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || p == nullptr) {
      (void)hipGetLastError();
      return RKV_ERR_HIP;
    }
    address[dev].store(p, std::memory_order_release);
  }
  *out = static_cast<char*>(p);
  return RKV_OK;
}

// An empty batch (num_problems == 0) is valid and enqueues nothing.
static bool empty(const Plan& pl) { return pl.heads == 0; }

}  // namespace rkv

using namespace rkv;

extern "C" {

rkv_status rkv_workspace_size(const rkv_params* prm, size_t* bytes) {
  if (bytes == nullptr) return RKV_ERR_NULL;
  Plan pl;
  const rkv_status s = make_plan(prm, &pl);
  if (s != RKV_OK) return s;
  *bytes = pl.total;
  return RKV_OK;
}

rkv_status rkv_score_importance(const rkv_params* prm, const void* q_obs, const void* k,
                                float* importance, void* ws, size_t ws_bytes, void* stream) {
  Plan pl;
  rkv_status s = make_plan(prm, &pl);
  if (s != RKV_OK) return s;
  if (empty(pl)) return RKV_OK;
  if (q_obs == nullptr || k == nullptr || importance == nullptr) return RKV_ERR_NULL;
  if ((s = check_ws(pl, ws, ws_bytes)) != RKV_OK) return s;
  hipStream_t st = static_cast<hipStream_t>(stream);
  char* w = static_cast<char*>(ws);
  if ((s = hip_status(launch_prepass(pl, q_obs, k, w, st))) != RKV_OK) return s;
  return hip_status(launch_finalize(pl, kModeImportance, w, nullptr, nullptr, importance, nullptr, nullptr,
                                    nullptr, nullptr, st));
}

rkv_status rkv_score_redundancy(const rkv_params* prm, const void* k, float* redundancy,
                                float* mean_sim, void* ws, size_t ws_bytes, void* stream) {
  Plan pl;
  rkv_status s = make_plan(prm, &pl);
  if (s != RKV_OK) return s;
  if (empty(pl)) return RKV_OK;
  if (k == nullptr || redundancy == nullptr) return RKV_ERR_NULL;
  if ((s = check_ws(pl, ws, ws_bytes)) != RKV_OK) return s;
  hipStream_t st = static_cast<hipStream_t>(stream);
  char* w = static_cast<char*>(ws);
  if ((s = hip_status(launch_prepass(pl, nullptr, k, w, st))) != RKV_OK) return s;
  if ((s = hip_status(launch_gram(pl, k, w, st))) != RKV_OK) return s;
  return hip_status(launch_finalize(pl, kModeRedundancy, w, nullptr, nullptr, nullptr, redundancy, mean_sim,
                                    nullptr, nullptr, st));
}

rkv_status rkv_select_topk(const rkv_params* prm, const float* importance, const float* redundancy,
                           float* score, int32_t* kept_idx, void* ws, size_t ws_bytes, void* stream) {
  Plan pl;
  rkv_status s = make_plan(prm, &pl);
  if (s != RKV_OK) return s;
  if (empty(pl)) return RKV_OK;
  if (importance == nullptr || redundancy == nullptr || kept_idx == nullptr) return RKV_ERR_NULL;
  if ((s = check_ws(pl, ws, ws_bytes)) != RKV_OK) return s;
  if (pl.N <= pl.budget) return RKV_NOT_TRIGGERED;
  hipStream_t st = static_cast<hipStream_t>(stream);
  char* w = static_cast<char*>(ws);
  if (!pl.shared_selection)
    return hip_status(launch_finalize(pl, kModeSelect, w, importance, redundancy, nullptr, nullptr, nullptr, score,
                                      kept_idx, st));
  if ((s = hip_status(launch_finalize(pl, kModeScore, w, importance, redundancy, nullptr, nullptr, nullptr, score,
                                      nullptr, st))) != RKV_OK)
    return s;
  return hip_status(launch_shared_select(pl, w, kept_idx, st));
}

rkv_status rkv_compact(const rkv_params* prm, const void* k, const void* v, const int32_t* kept_idx,
                       void* k_out, void* v_out, void* stream) {
  Plan pl;
  const rkv_status s = make_plan(prm, &pl);
  if (s != RKV_OK) return s;
  if (empty(pl)) return RKV_OK;
  if (k == nullptr || v == nullptr || kept_idx == nullptr || k_out == nullptr || v_out == nullptr) return RKV_ERR_NULL;
  return hip_status(launch_gather(pl, k, v, kept_idx, k_out, v_out, static_cast<hipStream_t>(stream)));
}

rkv_status rkv_compact_inplace(const rkv_params* prm, void* k, void* v, const int32_t* kept_idx, void* stream) {
  Plan pl;
  const rkv_status s = make_plan(prm, &pl);
  if (s != RKV_OK) return s;
  if (empty(pl)) return RKV_OK;
  if (k == nullptr || v == nullptr || kept_idx == nullptr) return RKV_ERR_NULL;
  return hip_status(launch_compact_inplace(pl, k, v, kept_idx, static_cast<hipStream_t>(stream)));
}

// `inplace` compacts inside k and v (k_out and v_out are then unused).
static rkv_status compress_impl(const rkv_params* prm, const void* q_obs, const void* k, const void* v,
                                void* k_out, void* v_out, int32_t* kept_idx, float* score,
                                void* ws, size_t ws_bytes, void* stream, void* const* events, bool inplace = false) {
  Plan pl;
  rkv_status s = make_plan(prm, &pl);
  if (s != RKV_OK) return s;
  if (empty(pl)) return RKV_OK;
  if (q_obs == nullptr || k == nullptr || v == nullptr) return RKV_ERR_NULL;
  if (!inplace && (k_out == nullptr || v_out == nullptr)) return RKV_ERR_NULL;
  if ((s = check_ws(pl, ws, ws_bytes)) != RKV_OK) return s;
  if (pl.N <= pl.budget) return RKV_NOT_TRIGGERED;
  hipStream_t st = static_cast<hipStream_t>(stream);
  char* w = static_cast<char*>(ws);
  int32_t* idx = kept_idx ? kept_idx : reinterpret_cast<int32_t*>(w + pl.off_idx);
  auto mark = [&](int i) -> rkv_status {
    if (events == nullptr) return RKV_OK;
    return hip_status(hipEventRecord(static_cast<hipEvent_t>(events[i]), st));
  };
  if ((s = mark(0)) != RKV_OK) return s;
  if ((s = hip_status(launch_prepass(pl, q_obs, k, w, st))) != RKV_OK) return s;
  if ((s = mark(1)) != RKV_OK) return s;
  // lambda == 1 makes Eq. 7 the importance score alone (attention-only eviction): the similarity
  // pass cannot influence the result and is not run.
  const bool attention_only = (pl.lambda == 1.0f);
  if (!attention_only && (s = hip_status(launch_gram(pl, k, w, st))) != RKV_OK) return s;
  if ((s = mark(2)) != RKV_OK) return s;
  const int pick = pl.shared_selection ? kModeScore : kModeSelect;
  const int mode = (attention_only ? kModeImportance : (kModeImportance | kModeRedundancy)) | pick;
  if ((s = hip_status(launch_finalize(pl, mode, w, nullptr, nullptr, nullptr, nullptr, nullptr, score, idx, st))) != RKV_OK)
    return s;
  if (pl.shared_selection && (s = hip_status(launch_shared_select(pl, w, idx, st))) != RKV_OK) return s;
  if ((s = mark(3)) != RKV_OK) return s;
  if (inplace) s = hip_status(launch_compact_inplace(pl, const_cast<void*>(k), const_cast<void*>(v), idx, st));
  else s = hip_status(launch_gather(pl, k, v, idx, k_out, v_out, st));
  if (s != RKV_OK) return s;
  return mark(4);
}

rkv_status rkv_compress_inplace(const rkv_params* prm, const void* q_obs, void* k, void* v, int32_t* kept_idx,
                                float* score, void* ws, size_t ws_bytes, void* stream) {
  return compress_impl(prm, q_obs, k, v, nullptr, nullptr, kept_idx, score, ws, ws_bytes, stream, nullptr, true);
}

rkv_status rkv_compress(const rkv_params* prm, const void* q_obs, const void* k, const void* v,
                        void* k_out, void* v_out, int32_t* kept_idx, float* score,
                        void* ws, size_t ws_bytes, void* stream) {
  return compress_impl(prm, q_obs, k, v, k_out, v_out, kept_idx, score, ws, ws_bytes, stream, nullptr);
}

rkv_status rkv_compress_static(const rkv_params* prm, const void* q_obs, const void* k, const void* v,
                               void* k_out, void* v_out, int32_t* kept_idx, float* score, void* stream) {
  // validate and size first: a shape whose scratch does not fit is refused before anything is looked up
  Plan pl;
  rkv_status s = make_plan(prm, &pl);
  if (s != RKV_OK) return s;
  if (empty(pl)) return RKV_OK;
  if (pl.total > (size_t)RKV_STATIC_SCRATCH_BYTES) return RKV_ERR_WORKSPACE;
  char* ws = nullptr;
  if (pl.N > pl.budget && (s = static_scratch(&ws)) != RKV_OK) return s;
  if (ws == nullptr) ws = reinterpret_cast<char*>(256);          // not triggered: never dereferenced
  return compress_impl(prm, q_obs, k, v, k_out, v_out, kept_idx, score, ws, (size_t)RKV_STATIC_SCRATCH_BYTES, stream, nullptr);
}

rkv_status rkv_compress_events(const rkv_params* prm, const void* q_obs, const void* k, const void* v,
                               void* k_out, void* v_out, int32_t* kept_idx, float* score,
                               void* ws, size_t ws_bytes, void* stream, void* const* events) {
  if (events == nullptr) return RKV_ERR_NULL;
  for (int i = 0; i < 5; ++i)
    if (events[i] == nullptr) return RKV_ERR_NULL;
  return compress_impl(prm, q_obs, k, v, k_out, v_out, kept_idx, score, ws, ws_bytes, stream, events);
}

rkv_status rkv_should_compress(const rkv_params* prm, int32_t cached_tokens) {
  Plan pl;
  const rkv_status s = make_plan(prm, &pl);
  if (s != RKV_OK) return s;
  // Alg. 1: compress once the rows held beyond the budget fill the buffer (here N = budget + buffer)
  return (cached_tokens >= pl.N && pl.N > pl.budget) ? RKV_OK : RKV_NOT_TRIGGERED;
}

rkv_status rkv_cache_append(const rkv_params* prm, void* k_cache, void* v_cache, void* q_cache,
                            const void* k_new, const void* v_new, const void* q_new,
                            int32_t position, int32_t q_slot, void* stream) {
  Plan pl;
  const rkv_status s = make_plan(prm, &pl);
  if (s != RKV_OK) return s;
  if (empty(pl)) return RKV_OK;
  if (k_cache == nullptr || v_cache == nullptr || q_cache == nullptr || k_new == nullptr || v_new == nullptr ||
      q_new == nullptr)
    return RKV_ERR_NULL;
  if (position < 0 || position >= pl.N || q_slot < 0 || q_slot >= pl.alpha) return RKV_ERR_SHAPE;
  return hip_status(launch_append(pl, k_cache, v_cache, q_cache, k_new, v_new, q_new, position, q_slot,
                                  static_cast<hipStream_t>(stream)));
}

const char* rkv_status_string(rkv_status s) {
  switch (s) {
    case RKV_OK: return "ok";
    case RKV_NOT_TRIGGERED: return "not triggered: the cache does not exceed the budget";
    case RKV_ERR_NULL: return "a required pointer is NULL";
    case RKV_ERR_SHAPE: return "inconsistent shape or strides";
    case RKV_ERR_UNSUPPORTED: return "shape outside the supported range";
    case RKV_ERR_WORKSPACE: return "workspace missing, misaligned or too small";
    case RKV_ERR_PARAM: return "hyper-parameter out of range";
    case RKV_ERR_HIP: return "HIP launch failure";
  }
  return "unknown status";
}

}  // extern "C"
