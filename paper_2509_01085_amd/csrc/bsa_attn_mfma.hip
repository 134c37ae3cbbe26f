// bf16 MFMA sparse attention kernels (placeholder until the kernels land).
#include "bsa_common.h"

namespace bsa {
bool mfma_supported(const Geom&, int, int) { return false; }
int launch_fwd_mfma(const Geom&, const AttnArgs&, hipStream_t) { return BSA_ERR_SHAPE; }
int launch_bwd_mfma(const Geom&, const AttnArgs&, hipStream_t) { return BSA_ERR_SHAPE; }
size_t bwd_workspace_mfma(const Geom&, int) { return 0; }
}  // namespace bsa
