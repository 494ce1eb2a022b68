// MFMA decode kernel for bf16 caches (placeholder until the tiled kernel lands).
#include "mlra_internal.h"

namespace mlra {
bool decode_mfma_supported(const DecodeArgs&) { return false; }
int launch_decode_mfma(const DecodeArgs&) { return MLRA_ERR_SHAPE; }
}  // namespace mlra
