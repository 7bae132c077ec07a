// Instantiation of the fused kernel for ceil(d / 32) = 2 (one file per value so
// that the variants compile in parallel).
#include "fused_impl.h"

namespace binattn {
template int launch_fused_dk<2>(const FusedParams &, int, hipStream_t);
template int launch_onehead_dk<2>(const FusedParams &, int, hipStream_t);
}
