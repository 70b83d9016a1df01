// placeholder until the MFMA backward lands
#include "launch.h"
namespace mate {
hipError_t launch_bwd_mfma(const AttnArgs& a, hipStream_t s) { return launch_bwd_scalar(a, true, s); }
}
