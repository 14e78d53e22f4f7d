// Host-side helpers shared by the launch code.
#pragma once
#include <hip/hip_runtime.h>

#include <atomic>

#include "metro.h"

namespace metro {

// Runs a set-up step once per device: kernel function attributes (such as the opt-in to more than 64 KB
// of dynamic LDS) belong to the device that is current when they are set.  Two threads racing on the
// first call both run the step, which is idempotent.
class PerDeviceOnce {
public:
    template <typename F>
    int run(F setup) {
        int dev = 0;
        if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return METRO_ERR_HIP;
        if (!done_[dev].load(std::memory_order_acquire)) {
            if (setup() != hipSuccess) return METRO_ERR_HIP;
            done_[dev].store(true, std::memory_order_release);
        }
        return METRO_OK;
    }

private:
    static constexpr int kMaxDevices = 64;
    std::atomic<bool> done_[kMaxDevices] = {};
};

}  // namespace metro
