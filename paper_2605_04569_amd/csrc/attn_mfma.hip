// MFMA attention kernels (bf16, D = 128, block = 128): placeholder until the kernels land.
#include "isa_internal.h"

namespace isa {
hipError_t launch_pack_vt(const Problem&, const Workspace&, const void*, hipStream_t) { return hipErrorNotSupported; }
hipError_t launch_gather_means(const Problem&, const Workspace&, const float*, const float*, const int*, hipStream_t) {
  return hipErrorNotSupported;
}
hipError_t launch_attn_mfma(const Problem&, const Workspace&, const AttnArgs&, hipStream_t) { return hipErrorNotSupported; }
}  // namespace isa
