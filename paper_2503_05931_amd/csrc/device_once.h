// Host-side helpers: set-up that has to happen once per device (function attributes of kernels with a large
// dynamic LDS size) and the device's number of compute units, safe to reach from several host threads and with
// several devices in one process.
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

// Workgroups of a persistent kernel that runs one workgroup per CU and deals its tiles out XCD by XCD: the current
// device's compute units rounded down to whole rounds over the 8 XCDs (256 on an unpartitioned MI355X), or the tiles
// rounded up to such rounds when there are fewer.  0: the device could not be asked.
inline int persistent_grid(int tiles) {
    static std::mutex mu;
    static int cus[64] = {};
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return 0;
    int n;
    {
        std::lock_guard<std::mutex> lock(mu);
        if (cus[dev] == 0) {
            int v = 0;
            if (hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || v < 8) return 0;
            cus[dev] = v / 8 * 8;
        }
        n = cus[dev];
    }
    return tiles >= n ? n : (tiles + 7) / 8 * 8;
}

}  // namespace aed
