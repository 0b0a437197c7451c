// Host-side helper: set-up that has to happen once per device (function attributes of kernels with a large
// dynamic LDS size), safe to reach from several host threads and with several devices in one process.
#pragma once

#include <hip/hip_runtime.h>

#include <mutex>

namespace aed {

class DeviceOnce {
public:
    // Runs f() with the current device unless it has already succeeded for that device.
    template <typename F> hipError_t run(F f) {
        int dev = 0;
        hipError_t e = hipGetDevice(&dev);
        if (e != hipSuccess) return e;
        if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
        std::lock_guard<std::mutex> lock(mu_);
        if (done_[dev]) return hipSuccess;
        e = f();
        if (e == hipSuccess) done_[dev] = true;
        return e;
    }

private:
    static constexpr int kMaxDevices = 64;
    std::mutex mu_;
    bool done_[kMaxDevices] = {};
};

}  // namespace aed
