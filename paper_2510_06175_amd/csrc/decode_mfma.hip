// Matrix-core decode attention (placeholder until the kernel lands).
#include "common.h"

namespace vecinfer {
bool decode_mfma_supports(const DecodeParams &) { return false; }
int launch_decode_mfma(const DecodeParams &, hipStream_t) { return -2; }
} // namespace vecinfer
