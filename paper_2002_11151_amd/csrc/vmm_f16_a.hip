// Contraction kernels on fp16 planes for crossbar tiles of up to 128 rows (two row patches per wave).
#include "vmm_device.h"

namespace xbar_detail {

hipError_t launch_vmm_f16_a(const VmmArgs& a, const VmmPlan& p, int terms, bool codes, hipStream_t st) {
  if (a.npol == 2) return launch_vmm_variant<2, 8, 2, true>(a, p, codes, st);   // planes of single arrays always come in two terms
  return terms == 2 ? launch_vmm_variant<2, 8, 2, false>(a, p, codes, st) : launch_vmm_variant<2, 8, 1, false>(a, p, codes, st);
}

}  // namespace xbar_detail
