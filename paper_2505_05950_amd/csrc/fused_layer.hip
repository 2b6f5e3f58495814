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

// The longest blocks (224 passes per producer wave = 896 channels per workgroup at d = 4096, then 112, 56, ... 7) that
// still give the chip about one workgroup per compute unit: every round of workgroups pays the kernel's prologue, the
// start of its streams and its tail again.  0 = do not fuse (too many partial results).
int fused_passes(int d, int f, int n_tasks, int max_tasks) {
    if (n_tasks <= 0 || n_tasks > max_tasks || n_tasks > kFusedMaxTasks) return 0;
    constexpr int n_options = sizeof(kFusedPassOptions) / sizeof(kFusedPassOptions[0]);
    int pick = kFusedPassOptions[n_options - 1];
    for (int i = 0; i < n_options; ++i) {
        if ((long long)fused_blocks(d, f, kFusedPassOptions[i]) * n_tasks >= 200 * fused_wgs_per_cu) {
            pick = kFusedPassOptions[i];
            break;
        }
    }
    return (long long)fused_blocks(d, f, pick) * n_tasks <= kFusedMaxWorkgroups ? pick : 0;
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
