// Contraction kernels on 6-bit planes with the full schedule of 5 terms (device variation, stored profile,
// all-paths wire model, arrays read one by one).
#include "vmm_device.h"

namespace xbar_detail {

hipError_t launch_vmm_f6_b(const VmmArgs& a, const VmmPlan& p, int terms, bool codes, hipStream_t st) {
  if (terms != 5) return hipErrorInvalidValue;
  return a.npol == 2 ? launch_vmm6_variant<5, true>(a, p, codes, st) : launch_vmm6_variant<5, false>(a, p, codes, st);
}

}  // namespace xbar_detail
