// Host side of the fused small-batch kernel: block-size choice and dispatch on the bit width.
#include "launch.h"

#include <atomic>

namespace floe {

int num_cus() {
    constexpr int kMaxDevices = 64, kDefault = 256;
    static std::atomic<int> cached[kMaxDevices];  // 0 = not asked yet
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return kDefault;
    int n = cached[dev].load(std::memory_order_relaxed);
    if (n > 0) return n;
    if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n <= 0) n = kDefault;
    cached[dev].store(n, std::memory_order_relaxed);
    return n;
}

static std::atomic<int> g_fused_tasks{0};
int fused_tasks_tuned() { return g_fused_tasks.load(std::memory_order_relaxed); }
void set_fused_tasks_tuned(int n) { g_fused_tasks.store(n > 0 ? n : 0, std::memory_order_relaxed); }

hipError_t launch_fused_int2(const FusedArgs& a, hipStream_t stream);
hipError_t launch_fused_int3(const FusedArgs& a, hipStream_t stream);
hipError_t launch_fused_int4(const FusedArgs& a, hipStream_t stream);

int fused_blocks(int d, int f, int passes) {
    const int ch = fused_producers * passes * (64 / (d / 64));
    return (f + ch - 1) / ch;
}

// Passes per producer wave such that the launch is about one workgroup per compute unit, all of them with the same
// number of channels: every round of workgroups pays the kernel's prologue, the start of its streams and its tail again,
// and a round that is not full leaves compute units idle.  0 = do not fuse.
int fused_passes(int d, int f, int bits, int n_tasks, int max_tasks) {
    if (n_tasks <= 0 || n_tasks > max_tasks || n_tasks > kFusedMaxTasks || f <= 0) return 0;
    const int unit = fused_producers * (64 / (d / 64));  // channels of one pass of all producers
    const int cus = num_cus() * fused_wgs_per_cu;
    int want_blocks = cus / n_tasks;  // rounded down: a few workgroups more than compute units cost a whole second round
    if (want_blocks < 1) want_blocks = 1;
    const int per_block = (f + want_blocks - 1) / want_blocks;
    int passes = (per_block + unit - 1) / unit;
    if (passes <= kFusedMinPasses) {
        passes = kFusedMinPasses;
    } else if (bits == 2) {  // staged codes: whole rounds of the ring
        const int depth = fused_depth(d, bits);
        passes = (passes + depth - 1) / depth * depth;
    }
    if (passes > kFusedMaxPasses) passes = kFusedMaxPasses / 14 * 14;
    return (long long)fused_blocks(d, f, passes) * n_tasks <= kFusedMaxWorkgroups ? passes : 0;
}

hipError_t launch_fused(const FusedArgs& a, int bits, hipStream_t stream) {
    switch (bits) {
        case 2: return launch_fused_int2(a, stream);
        case 3: return launch_fused_int3(a, stream);
        case 4: return launch_fused_int4(a, stream);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace floe
