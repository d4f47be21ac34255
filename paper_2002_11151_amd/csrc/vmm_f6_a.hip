// Contraction kernels on 6-bit planes with 1 term (ideal arrays) or 4 terms (single-path wire model alone).
#include "vmm_device.h"

namespace xbar_detail {

hipError_t launch_vmm_f6_a(const VmmArgs& a, const VmmPlan& p, int terms, bool codes, hipStream_t st) {
  if (a.npol != 1) return hipErrorInvalidValue;
  switch (terms) {
    case 1: return launch_vmm6_variant<1, false>(a, p, codes, st);
    case 4: return launch_vmm6_variant<4, false>(a, p, codes, st);
    default: return hipErrorInvalidValue;
  }
}

}  // namespace xbar_detail
