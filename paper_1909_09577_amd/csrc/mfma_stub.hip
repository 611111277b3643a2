#include "nm_common.h"
namespace nm {
bool mfma_fwd_supported(const Geom &) { return false; }
size_t mfma_fwd_workspace(const Geom &) { return 0; }
hipError_t launch_mfma_fwd(const Geom &, const void *, const void *, const float *, const float *, const void *, void *, bool, void *, hipStream_t) { return hipErrorNotSupported; }
bool mfma_dgrad_supported(const Geom &) { return false; }
size_t mfma_dgrad_workspace(const Geom &) { return 0; }
hipError_t launch_mfma_dgrad(const Geom &, const void *, const void *, const float *, const void *, void *, void *, bool, void *, hipStream_t) { return hipErrorNotSupported; }
bool mfma_wgrad_supported(const Geom &) { return false; }
size_t mfma_wgrad_workspace(const Geom &, bool) { return 0; }
hipError_t launch_mfma_wgrad(const Geom &, const void *, const void *, const void *, const float *, float *, bool, bool, void *, hipStream_t) { return hipErrorNotSupported; }
}
