// Search kernels with the run-time switches folded away, eight expansions per step (see search_kernel.hpp).
#include "search_kernel.hpp"

namespace ann {
ann_status launch_search_fast_wide(const SearchArgs &a, uint32_t bits, uint32_t lpr, int m, hipStream_t st) {
  return launch_search<true, true>(a, bits, lpr, m, true, st);
}
}  // namespace ann
