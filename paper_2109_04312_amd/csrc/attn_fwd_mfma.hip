// placeholder until the MFMA forward lands
#include "launch.h"
namespace mate {
hipError_t launch_fwd_mfma(const AttnArgs& a, hipStream_t s) { return launch_fwd_scalar(a, true, s); }
}
