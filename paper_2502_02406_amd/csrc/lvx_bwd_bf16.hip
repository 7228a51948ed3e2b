#include "lvx_internal.h"
namespace lvx {
int bwd_bf16_pick_split(const Dims&, int) { return 1; }
hipError_t launch_bwd_bf16(const BwdArgs&, hipStream_t) { return hipErrorNotSupported; }
}
