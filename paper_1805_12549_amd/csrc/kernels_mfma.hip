// Matrix-core (MFMA) kernels for the gated convolution: placeholder plan that
// declines every shape until the kernels land.
#include "cg_device.h"

namespace cg {

MfmaPlan mfma_plan(const cg_conv_desc& d) {
  (void)d;
  MfmaPlan p{};
  p.ok = 0;
  return p;
}

hipError_t launch_mfma_pack(const MfmaPlan&, const Params&, void*, void*, hipStream_t) { return hipErrorNotSupported; }
hipError_t launch_mfma(const MfmaPlan&, const Params&, const void*, const void*, hipStream_t) {
  return hipErrorNotSupported;
}

}  // namespace cg
