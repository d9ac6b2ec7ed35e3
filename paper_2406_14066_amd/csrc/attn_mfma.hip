// placeholder until the matrix-instruction kernel lands
#include "common.h"
namespace specv {
hipError_t launch_attn_mfma(const AttnParams &, int, hipStream_t) { return hipErrorNotSupported; }
}
