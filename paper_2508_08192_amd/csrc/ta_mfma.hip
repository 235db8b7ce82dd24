// placeholder until the matrix-core kernel lands
#include "ta_common.h"
hipError_t ta_launch_mfma(const TAParams &p, hipStream_t stream) { return ta_launch_generic(p, stream); }
