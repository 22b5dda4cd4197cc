// placeholder until the MFMA kernels land
#include "citrus_internal.h"
namespace citrus {
bool mfma_path_supported(int, const Dims&) { return false; }
hipError_t launch_attn_mfma(const Dims&, View, int, Segments, Segments, int, View, float*, hipStream_t) { return hipErrorNotSupported; }
hipError_t launch_colsum_mfma(const Dims&, View, int, Segments, int, const float*, float*, hipStream_t) { return hipErrorNotSupported; }
}
