// The fused small-batch kernel (fused_ffn.h) for INT4 codes.
#include "fused_ffn.h"

namespace floe {

hipError_t launch_fused_int4(const FusedArgs& a, hipStream_t stream) { return fused_launch_bits<4>(a, stream); }

}  // namespace floe
