// Fused two-stage chain (intermediate kept in LDS) -- bf16, R <= 512.
#include "sk_launch.h"

namespace sk {

bool chain_supported(int) { return false; }
int chain_bm(int) { return 0; }
hipError_t launch_chain_bf16(bool, const ChainArgs&, hipStream_t) { return hipErrorNotSupported; }

}  // namespace sk
