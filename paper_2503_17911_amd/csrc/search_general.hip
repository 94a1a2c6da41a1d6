// Search kernels that take every switch at run time (see search_kernel.hpp).
#include "search_kernel.hpp"

namespace ann {
ann_status launch_search_general(const SearchArgs &a, uint32_t bits, uint32_t lpr, int m, bool multi, hipStream_t st) {
  return launch_search<false, false>(a, bits, lpr, m, multi, st);
}
}  // namespace ann
