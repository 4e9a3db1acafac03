// One addressing mode of the DCT axis pass (see mfma_dct_impl.h); split per mode so the variants build in parallel.
#include "mfma_dct_impl.h"

namespace fa {
hipError_t launch_mfma_dct_scatter(const DctPassArgs& a, int num_cu, hipStream_t st, int* waves_out) {
  return dispatch_mode<2>(a, num_cu, st, waves_out);
}
}  // namespace fa
