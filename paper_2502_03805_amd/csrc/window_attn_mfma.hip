// Observation-window attention on the matrix cores (placeholder until the kernels land).
#include "common.hpp"
namespace ckv {
bool attn_mfma_supported(const Dims &) { return false; }
int mfma_attn_chunks(const Dims &d) { return generic_attn_chunks(d); }
hipError_t launch_attn_stats_mfma(const Dims &, const void *, const void *, float *, int, hipStream_t) { return hipErrorNotSupported; }
hipError_t launch_attn_colsum_mfma(const Dims &, const void *, const void *, const float *, float *, hipStream_t) { return hipErrorNotSupported; }
} // namespace ckv
