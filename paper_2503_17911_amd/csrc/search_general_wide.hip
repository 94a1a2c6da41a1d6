// Search kernels that take every switch at run time, up to eight expansions per step (see search_kernel.hpp).
#include "search_kernel.hpp"

namespace ann {
ann_status launch_search_general_wide(const SearchArgs &a, uint32_t bits, uint32_t lpr, int m, hipStream_t st) {
  return launch_search<false, true>(a, bits, lpr, m, true, st);
}
}  // namespace ann
