// Kernel A of the compress path for bf16 storage (see compress_gq16.h).
#include "compress_gq16.h"

namespace lsp {
hipError_t launch_gq16_bf16(const CompressGroup& g, int32_t r, int32_t d, int blocks_per_wg, hipStream_t st) {
    return launch_gq16<BF16>(g, r, d, blocks_per_wg, st);
}
}  // namespace lsp

#ifdef LSP_PHASE_TIMING
// copies the per-wave phase sums of the last bf16 kernel A launches (this translation unit's copy of the array) to
// host memory (development builds only)
extern "C" int lsp_dev_phase_read(void* host, size_t bytes) {
    return (int)hipMemcpyFromSymbol(host, HIP_SYMBOL(lsp::g_phase), bytes, 0, hipMemcpyDeviceToHost);
}
#endif
