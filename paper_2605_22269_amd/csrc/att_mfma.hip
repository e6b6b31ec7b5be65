// Eq. 1 on the matrix cores (bf16 payload, D = 128).  Placeholder until the MFMA kernel lands.
#include "mukv_internal.h"

namespace mukv {

hipError_t launch_att_mfma(const Ctx &, const ChunkArgs &, float *, int *, hipStream_t) { return hipErrorNotSupported; }

} // namespace mukv
