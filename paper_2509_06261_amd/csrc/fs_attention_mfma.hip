// MFMA split-K paged decode-attention kernel (placeholder until the tuned kernel lands).
#include "fs_attention.h"

namespace fs {

bool mfma_supports(const DevBatch&) { return false; }

hipError_t launch_mfma(const MultiArgs&, int, hipStream_t) { return hipErrorNotSupported; }

}  // namespace fs
