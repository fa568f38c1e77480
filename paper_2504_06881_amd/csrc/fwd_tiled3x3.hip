// placeholder until the tiled kernel lands
#include "tconv_internal.h"
namespace tconv {
bool forward_tiled3x3_supported(const Params&, int) { return false; }
hipError_t launch_forward_tiled3x3(const Params&, int, const FwdArgs&, hipStream_t) { return hipErrorNotSupported; }
}
