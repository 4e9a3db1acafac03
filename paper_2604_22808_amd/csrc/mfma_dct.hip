// Dispatcher of the DCT axis pass (paper sections 3.2, 3.7): picks the addressing mode of the launch; the kernel is in
// mfma_dct_impl.h and is instantiated once per mode in mfma_dct_<mode>.hip.
#include <hip/hip_runtime.h>

#include "ctx.h"

namespace fa {

hipError_t launch_mfma_dct_plain(const DctPassArgs& a, int num_cu, hipStream_t st, int* waves_out);
hipError_t launch_mfma_dct_plain_tot(const DctPassArgs& a, int num_cu, hipStream_t st, int* waves_out);
hipError_t launch_mfma_dct_scatter(const DctPassArgs& a, int num_cu, hipStream_t st, int* waves_out);
hipError_t launch_mfma_dct_scatter_en(const DctPassArgs& a, int num_cu, hipStream_t st, int* waves_out);
hipError_t launch_mfma_dct_gather(const DctPassArgs& a, int num_cu, hipStream_t st, int* waves_out);

bool mfma_dct_supported(int n_in, int n_out) {
  if (n_in % 16 || n_in < 16 || n_in > 128 || n_out < 1 || n_out > 128) return false;
  const bool pow2 = n_in == 16 || n_in == 32 || n_in == 64 || n_in == 128;
  if (pow2) return true;                      // any number of output tiles
  return (n_out + 31) / 32 == (n_in + 31) / 32;  // other lengths: square passes only
}

hipError_t launch_mfma_dct_pass(const DctPassArgs& a, int num_cu, hipStream_t st, int* waves_out) {
  if (a.inner % 64 != 0 || a.inner % a.d != 0 || !mfma_dct_supported(a.n, a.n_out) || a.ldm < a.n) return hipErrorInvalidValue;
  if (a.perm_in && a.perm_out) return hipErrorInvalidValue;
  if (a.perm_in) return (a.masks && a.in_alt) ? launch_mfma_dct_gather(a, num_cu, st, waves_out) : hipErrorInvalidValue;
  if (a.perm_out) return a.energy_part ? launch_mfma_dct_scatter_en(a, num_cu, st, waves_out)
                                       : launch_mfma_dct_scatter(a, num_cu, st, waves_out);
  if (a.energy_part) return hipErrorInvalidValue;
  return a.tot_part ? launch_mfma_dct_plain_tot(a, num_cu, st, waves_out) : launch_mfma_dct_plain(a, num_cu, st, waves_out);
}

}  // namespace fa
