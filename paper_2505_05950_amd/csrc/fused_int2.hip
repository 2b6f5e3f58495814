// The fused small-batch kernel (fused_ffn.h) for INT2 codes.
#include "fused_ffn.h"

namespace floe {

hipError_t launch_fused_int2(const FusedArgs& a, hipStream_t stream) { return fused_launch_bits<2>(a, stream); }

#ifdef FLOE_TIMELINE
extern "C" int floe_debug_set_timeline_fused(unsigned long long* p) {
    return (int)hipMemcpyToSymbol(HIP_SYMBOL(g_timeline), &p, sizeof(p));
}
#endif

}  // namespace floe
