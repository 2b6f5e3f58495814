// The fused small-batch kernel (fused_ffn.h) for INT3 codes.
#include "fused_ffn.h"

namespace floe {

hipError_t launch_fused_int3(const FusedArgs& a, hipStream_t stream) { return fused_launch_bits<3>(a, stream); }

}  // namespace floe
