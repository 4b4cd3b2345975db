// placeholder until the MFMA kernels land
#include "kparams.h"
namespace ssa {
bool mfma_supported(const KP&, bool) { return false; }
hipError_t launch_mfma_fwd(const KP&, bool, hipStream_t) { return hipErrorNotSupported; }
hipError_t launch_mfma_dq(const KP&, hipStream_t) { return hipErrorNotSupported; }
hipError_t launch_mfma_dkdv(const KP&, hipStream_t) { return hipErrorNotSupported; }
hipError_t launch_mfma_dbias(const KP&, hipStream_t) { return hipErrorNotSupported; }
}
