// Tree-masked attention on the matrix cores (bf16 in, fp32 accumulate).  Placeholder until the
// MFMA kernel lands: no shape is routed here yet.
#include "common.h"

namespace s4c {

bool mfma_path_supported(const s4c_attn_shape&) { return false; }
int mfma_rows_per_block(const s4c_attn_shape&) { return 64; }
hipError_t launch_tree_attn_mfma(const AttnArgs&, hipStream_t) { return hipErrorNotSupported; }

}  // namespace s4c
