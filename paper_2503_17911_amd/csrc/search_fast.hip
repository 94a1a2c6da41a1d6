// Search kernels with the run-time switches folded away (see search_kernel.hpp).
#include "search_kernel.hpp"

namespace ann {
ann_status launch_search_fast(const SearchArgs &a, uint32_t bits, uint32_t lpr, int m, bool multi, hipStream_t st) {
  return launch_search<true, false>(a, bits, lpr, m, multi, st);
}
}  // namespace ann
