// Shared by the C ABI translation units: error reporting and device selection.
#pragma once
#include <hip/hip_runtime.h>

#include <string>

namespace tns {

// Record the detail of a failure for tns_last_error() (per thread) and return `code`.
int fail(int code, const std::string& msg);
int fail_hip(hipError_t e, const char* what);
void clear_error();

// Switches to a device for the lifetime of the object and restores the caller's.
class DeviceGuard {
public:
    explicit DeviceGuard(int dev) {
        ok_ = hipGetDevice(&prev_) == hipSuccess;
        if (ok_ && prev_ != dev) {
            err_ = hipSetDevice(dev);
            switched_ = err_ == hipSuccess;
        }
        if (!ok_) err_ = hipErrorNoDevice;
    }
    ~DeviceGuard() {
        if (switched_) (void)hipSetDevice(prev_);
    }
    hipError_t error() const { return err_; }

private:
    int prev_ = 0;
    bool ok_ = false, switched_ = false;
    hipError_t err_ = hipSuccess;
};

}  // namespace tns
