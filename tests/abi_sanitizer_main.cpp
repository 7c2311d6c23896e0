// Host-side validation of librkv under AddressSanitizer and UndefinedBehaviorSanitizer (host code only):
// every entry point is called with shapes, strides, flags and pointers that must be refused (or accepted)
// before anything is launched, and the size query is swept over a grid of shapes.  No GPU is needed: calls
// that would launch are made only with arguments that fail validation first.  Prints "ok <calls>" on success.
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <initializer_list>

#include "rkv.h"

static long calls = 0;
#define EXPECT(expr, want)                                                                   \
  do {                                                                                       \
    const int got_ = (int)(expr);                                                            \
    ++calls;                                                                                 \
    if (got_ != (int)(want)) {                                                               \
      std::printf("line %d: %s = %d (%s), expected %d\n", __LINE__, #expr, got_, rkv_status_string((rkv_status)got_), (int)(want)); \
      std::exit(1);                                                                          \
    }                                                                                        \
  } while (0)

static rkv_params base() {
  rkv_params p;
  std::memset(&p, 0, sizeof p);
  p.num_problems = 2; p.kv_heads = 8; p.q_heads = 32; p.n_tokens = 1152; p.head_dim = 128; p.alpha = 8;
  p.budget = 1024; p.pool_w = 4; p.beta = 1; p.sim_threshold = 0.5f; p.lambda = 0.1f; p.eps = 1e-8f;
  return p;
}

int main() {
  void* fake = reinterpret_cast<void*>(0x1000);          // never dereferenced: validation fails first
  size_t bytes = 0;
  rkv_params p = base();
  EXPECT(rkv_workspace_size(&p, &bytes), RKV_OK);
  EXPECT(rkv_workspace_size(nullptr, &bytes), RKV_ERR_NULL);
  EXPECT(rkv_workspace_size(&p, nullptr), RKV_ERR_NULL);
  // a grid of shapes: every combination either sizes a workspace or is refused with a status, never more
  const int ns[] = {2, 9, 10, 64, 65, 129, 1000, 1152, 4224, 8320, 32768, 32769, 1 << 30};
  const int alphas[] = {0, 1, 8, 16, 63, 64, 65};
  const int groups[] = {1, 2, 5, 8, 9, 64};
  const int betas[] = {-1, 0, 1, 2, 1 << 30};
  const int ws_[] = {-1, 0, 4, 1000, 1001, 1 << 30};
  const int Ps[] = {-1, 0, 1, 32, 768, 1 << 22, 1 << 30};
  for (int n : ns) for (int al : alphas) for (int g : groups) for (int b : betas) for (int w : ws_) for (int P : Ps)
    for (uint32_t flags : {0u, 1u, 2u, 4u, 8u, 16u, 24u, 32u, 63u, 64u, 0x80000000u}) {
      rkv_params q = base();
      q.n_tokens = n; q.alpha = al; q.q_heads = q.kv_heads * g; q.beta = b; q.pool_w = w; q.num_problems = P; q.flags = flags;
      q.budget = n / 2 + 1;
      bytes = 0;
      const int s = rkv_workspace_size(&q, &bytes);
      ++calls;
      if (s > 0 || s < RKV_ERR_HIP || (s == RKV_OK && P > 0 && bytes == 0)) { std::printf("unexpected status %d\n", s); return 1; }
    }
  // strides
  p = base();
  p.k_stride_token = 100; p.k_stride_head = 8; p.k_stride_problem = 8;
  EXPECT(rkv_workspace_size(&p, &bytes), RKV_ERR_SHAPE);
  p = base();
  p.q_stride_problem = 8 * 32 * 128; p.q_stride_head = 128; p.q_stride_token = 32 * 128;
  EXPECT(rkv_workspace_size(&p, &bytes), RKV_OK);
  p.q_stride_token = INT64_MAX - 7;                       // absurd but aligned: accepted by the size query, never multiplied on the host
  EXPECT(rkv_workspace_size(&p, &bytes) <= 0, 1);
  // paged caches
  p = base();
  p.page_size = 16; p.table_stride = 72; p.block_table = reinterpret_cast<const int32_t*>(fake);
  p.k_stride_page = p.v_stride_page = 8 * 16 * 128; p.k_stride_head = p.v_stride_head = 16 * 128;
  p.k_stride_token = p.v_stride_token = 128;
  EXPECT(rkv_workspace_size(&p, &bytes), RKV_OK);
  p.table_stride = 71;
  EXPECT(rkv_workspace_size(&p, &bytes), RKV_ERR_SHAPE);
  p.table_stride = INT32_MAX; p.page_size = 128;
  EXPECT(rkv_workspace_size(&p, &bytes), RKV_OK);
  // compute entry points: refused before any launch
  p = base();
  EXPECT(rkv_compress(&p, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, 0, nullptr), RKV_ERR_NULL);
  EXPECT(rkv_compress(&p, fake, fake, fake, fake, fake, nullptr, nullptr, nullptr, 0, nullptr), RKV_ERR_WORKSPACE);
  EXPECT(rkv_compress(&p, fake, fake, fake, fake, fake, nullptr, nullptr, reinterpret_cast<void*>(0x1001), SIZE_MAX, nullptr), RKV_ERR_WORKSPACE);
  EXPECT(rkv_compress(&p, fake, fake, fake, fake, fake, nullptr, nullptr, fake, 16, nullptr), RKV_ERR_WORKSPACE);
  EXPECT(rkv_compress_inplace(&p, fake, nullptr, fake, nullptr, nullptr, fake, SIZE_MAX, nullptr), RKV_ERR_NULL);
  EXPECT(rkv_score_importance(&p, fake, fake, nullptr, fake, SIZE_MAX, nullptr), RKV_ERR_NULL);
  EXPECT(rkv_score_redundancy(&p, fake, nullptr, nullptr, fake, SIZE_MAX, nullptr), RKV_ERR_NULL);
  EXPECT(rkv_select_topk(&p, static_cast<const float*>(fake), static_cast<const float*>(fake), nullptr, nullptr, fake, SIZE_MAX, nullptr), RKV_ERR_NULL);
  EXPECT(rkv_compact(&p, fake, fake, nullptr, fake, fake, nullptr), RKV_ERR_NULL);
  EXPECT(rkv_compact_inplace(&p, fake, fake, nullptr, nullptr), RKV_ERR_NULL);
  EXPECT(rkv_compress_events(&p, fake, fake, fake, fake, fake, nullptr, nullptr, fake, SIZE_MAX, nullptr, nullptr), RKV_ERR_NULL);
  EXPECT(rkv_cache_append(&p, fake, fake, fake, fake, fake, fake, 1152, 0, nullptr), RKV_ERR_SHAPE);
  EXPECT(rkv_cache_append(&p, fake, fake, fake, fake, fake, fake, 0, 8, nullptr), RKV_ERR_SHAPE);
  rkv_params calm = base();
  calm.n_tokens = 1024;
  EXPECT(rkv_compress(&calm, fake, fake, fake, fake, fake, nullptr, nullptr, fake, SIZE_MAX, nullptr), RKV_NOT_TRIGGERED);
  EXPECT(rkv_compress_static(&calm, fake, fake, fake, fake, fake, nullptr, nullptr, nullptr), RKV_NOT_TRIGGERED);
  EXPECT(rkv_should_compress(&p, 1152), RKV_OK);
  EXPECT(rkv_should_compress(&p, 1151), RKV_NOT_TRIGGERED);
  rkv_params big = base();
  big.num_problems = 32; big.n_tokens = 4224; big.budget = 4096;
  EXPECT(rkv_compress_static(&big, fake, fake, fake, fake, fake, nullptr, nullptr, nullptr), RKV_ERR_WORKSPACE);
  rkv_params none = base();
  none.num_problems = 0;
  EXPECT(rkv_compress(&none, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, 0, nullptr), RKV_OK);
  for (int s = -7; s <= 2; ++s) { if (rkv_status_string((rkv_status)s) == nullptr) return 1; ++calls; }
  std::printf("ok %ld\n", calls);
  return 0;
}
