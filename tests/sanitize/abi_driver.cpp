// Calls the library's C ABI with arguments that must be refused on the host
// (no GPU work is started).  Linked against a host-only build of the library
// with -fsanitize=address,undefined by tests/test_sanitizers.py.
#include <stdio.h>
#include <string.h>

#include "ann.h"

static int failures = 0;
#define EXPECT(call, want)                                                        \
  do {                                                                            \
    ann_status got_ = (call);                                                     \
    if (got_ != (want)) {                                                         \
      printf("%s: got %d, want %d (%s)\n", #call, (int)got_, (int)(want), ann_last_error()); \
      ++failures;                                                                 \
    }                                                                             \
  } while (0)

int main() {
  ann_index *ix = nullptr;
  ann_index_desc d;
  memset(&d, 0, sizeof(d));
  float f[8] = {0};
  uint32_t u[8] = {0};
  uint8_t b[8] = {0};
  EXPECT(ann_upload_index(nullptr, nullptr, &ix), ANN_EINVAL);
  EXPECT(ann_upload_index(&d, nullptr, nullptr), ANN_EINVAL);
  EXPECT(ann_upload_index(&d, nullptr, &ix), ANN_EINVAL);
  d.n = 10, d.d = 4, d.degree = 200, d.metric = ANN_L2, d.n_levels = 1;
  EXPECT(ann_upload_index(&d, nullptr, &ix), ANN_ECAPACITY);
  d.degree = 2, d.adjacency = u, d.level[0].bits = 4, d.d = 5;
  d.level[0].codes = b, d.level[0].lo = f, d.level[0].delta = f, d.level[0].norm_term = f;
  EXPECT(ann_upload_index(&d, nullptr, &ix), ANN_EINVAL);   /* odd d with 4-bit codes */
  d.d = 4, d.level[0].norm_term = nullptr;
  EXPECT(ann_upload_index(&d, nullptr, &ix), ANN_EINVAL);   /* L2 without norm terms */
  d.level[0].norm_term = f, d.flags = ANN_DESC_UNIT_NORM_L2_KEYS;
  EXPECT(ann_upload_index(&d, nullptr, &ix), ANN_EINVAL);   /* the flag is for inner-product indexes */
  d.flags = 0, d.entry_point = 10;
  EXPECT(ann_upload_index(&d, nullptr, &ix), ANN_EINVAL);
  ann_search_params p;
  memset(&p, 0, sizeof(p));
  p.k = 10, p.ef = 5;
  EXPECT(ann_search_batch(nullptr, f, 1, &p, nullptr, 0, u, nullptr, nullptr, nullptr, nullptr), ANN_EINVAL);
  EXPECT(ann_search_batch_static(nullptr, f, 1, &p, nullptr, 0, u, nullptr, nullptr, nullptr, nullptr), ANN_EINVAL);
  EXPECT(ann_rerank(nullptr, f, 1, u, 1, 1, 1, u, f, nullptr), ANN_EINVAL);
  EXPECT(ann_rerank_adaptive(nullptr, f, 1, u, f, 1, 1, 1, 0.5f, 1, u, f, nullptr, nullptr), ANN_EINVAL);
  EXPECT(ann_rescore(nullptr, 0, f, 1, u, 1, 1, u, nullptr, nullptr, nullptr), ANN_EINVAL);
  EXPECT(ann_query_prep(nullptr, 0, f, 1, nullptr, nullptr, nullptr, nullptr), ANN_EINVAL);
  EXPECT(ann_entry_scan(nullptr, f, 1, 1, u, nullptr), ANN_EINVAL);
  EXPECT(ann_build_entry_table(nullptr, 4, nullptr), ANN_EINVAL);
  EXPECT(ann_build_prs(nullptr, nullptr), ANN_EINVAL);
  EXPECT(ann_reserve_workspace(nullptr, 4, nullptr), ANN_EINVAL);
  EXPECT(ann_schedule_queries(nullptr, 4, 4, u, nullptr), ANN_EINVAL);
  EXPECT(ann_bruteforce_topk(f, 100, 8, f, 1, 300, 0, u, f, nullptr), ANN_ECAPACITY);
  EXPECT(ann_sq_encode(f, 10, 5, 4, f, f, b, f, nullptr), ANN_EINVAL);
  EXPECT(ann_sq_train(nullptr, 10, 4, 8, f, f, nullptr), ANN_EINVAL);
  EXPECT(ann_sq_train_truncated(f, 10, 4, 8, 0.2, f, f, nullptr), ANN_EINVAL);
  EXPECT(ann_free_index(nullptr), ANN_OK);
  printf("%s: %d unexpected results\n", ann_version(), failures);
  return failures;
}
